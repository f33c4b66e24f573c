// Gathers the per-(dtype, layout) MFMA tile tables into one list.
#include "common.hpp"

namespace optiml {

const Variant *kTile_f32_rr(), *kTile_f32_rc(), *kTile_f32_cr(), *kTile_f32_cc();
const Variant *kTile_bf16_rr(), *kTile_bf16_rc(), *kTile_bf16_cr(), *kTile_bf16_cc();
const Variant *kDirect_bf16_rr(), *kDirect_bf16_rc();
const Variant *kRing_bf16_rr(), *kRing_bf16_rc();
const Variant *kRing_f32_rr(), *kRing_f32_rc();

namespace {
struct Gather {
    Variant v[8 * kTilesPerUnit + 2 * kDirectPerUnit + 2 * kRingPerUnit + 2 * kRingF32PerUnit];
    Gather()
    {
        // the direct-to-LDS kernels come first: where they apply the dispatcher prefers them
        constexpr int R = 2 * kRingPerUnit, F = R + 2 * kDirectPerUnit, D = F + 2 * kRingF32PerUnit;
        for (int i = 0; i < kRingF32PerUnit; ++i) {
            v[F + i] = kRing_f32_rr()[i];
            v[F + kRingF32PerUnit + i] = kRing_f32_rc()[i];
        }
        for (int i = 0; i < kRingPerUnit; ++i) {
            v[i] = kRing_bf16_rr()[i];
            v[kRingPerUnit + i] = kRing_bf16_rc()[i];
        }
        for (int i = 0; i < kDirectPerUnit; ++i) {
            v[R + i] = kDirect_bf16_rr()[i];
            v[R + kDirectPerUnit + i] = kDirect_bf16_rc()[i];
        }
        const Variant *units[8] = {kTile_f32_rr(),  kTile_f32_rc(),  kTile_f32_cr(),  kTile_f32_cc(),
                                   kTile_bf16_rr(), kTile_bf16_rc(), kTile_bf16_cr(), kTile_bf16_cc()};
        for (int u = 0; u < 8; ++u)
            for (int i = 0; i < kTilesPerUnit; ++i) v[D + u * kTilesPerUnit + i] = units[u][i];
    }
};
}  // namespace

const Variant *tile_variants()
{
    static const Gather g;
    return g.v;
}
const int kNumTileVariants = 8 * kTilesPerUnit + 2 * kDirectPerUnit + 2 * kRingPerUnit + 2 * kRingF32PerUnit;

}  // namespace optiml
