// Gathers the per-(dtype, layout) MFMA tile tables into one list.
#include "common.hpp"

namespace optiml {

const Variant *kTile_f32_rr(), *kTile_f32_rc(), *kTile_f32_cr(), *kTile_f32_cc();
const Variant *kTile_bf16_rr(), *kTile_bf16_rc(), *kTile_bf16_cr(), *kTile_bf16_cc();
const Variant *kTile_f16_rr(), *kTile_f16_rc(), *kTile_f16_cr(), *kTile_f16_cc();
const Variant *kDirect_bf16_rr(), *kDirect_bf16_rc(), *kDirect_f16_rr(), *kDirect_f16_rc();
const Variant *kRing_bf16_rr(), *kRing_bf16_rc(), *kRing_f16_rr(), *kRing_f16_rc(), *kRing_f8_rc(), *kRing_f4_rc(), *kRing_bf8_rc();
const Variant *kRing_f32_rr(), *kRing_f32_rc();

namespace {
constexpr int kTotal = 12 * kTilesPerUnit + 4 * kDirectPerUnit + 7 * kRingPerUnit + 2 * kRingF32PerUnit;
struct Gather {
    Variant v[kTotal];
    Gather()
    {
        // order = the dispatcher's preference where several apply: ring kernels, then the
        // direct-to-LDS ones, then the staged tiles
        int n = 0;
        auto add = [&](const Variant *unit, int count) {
            for (int i = 0; i < count; ++i) v[n++] = unit[i];
        };
        add(kRing_bf16_rr(), kRingPerUnit);
        add(kRing_bf16_rc(), kRingPerUnit);
        add(kDirect_bf16_rr(), kDirectPerUnit);
        add(kDirect_bf16_rc(), kDirectPerUnit);
        add(kRing_f32_rr(), kRingF32PerUnit);
        add(kRing_f32_rc(), kRingF32PerUnit);
        const Variant *units[8] = {kTile_f32_rr(),  kTile_f32_rc(),  kTile_f32_cr(),  kTile_f32_cc(),
                                   kTile_bf16_rr(), kTile_bf16_rc(), kTile_bf16_cr(), kTile_bf16_cc()};
        for (int u = 0; u < 8; ++u) add(units[u], kTilesPerUnit);
        // fp16 after everything that existed before it, so that variant indices stay put
        add(kRing_f16_rr(), kRingPerUnit);
        add(kRing_f16_rc(), kRingPerUnit);
        add(kDirect_f16_rr(), kDirectPerUnit);
        add(kDirect_f16_rc(), kDirectPerUnit);
        add(kTile_f16_rr(), kTilesPerUnit);
        add(kTile_f16_rc(), kTilesPerUnit);
        add(kTile_f16_cr(), kTilesPerUnit);
        add(kTile_f16_cc(), kTilesPerUnit);
        add(kRing_f8_rc(), kRingPerUnit);
        add(kRing_bf8_rc(), kRingPerUnit);
        add(kRing_f4_rc(), kRingPerUnit);
    }
};
}  // namespace

const Variant *tile_variants()
{
    static const Gather g;
    return g.v;
}
const int kNumTileVariants = kTotal;

}  // namespace optiml
