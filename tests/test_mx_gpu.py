"""The contraction on block-scaled (microscaling) E2M1, E4M3, E5M2, E2M3 and E3M2 operands against the CPU oracle, through the C-ABI.

Bar.  Every product a b is exact, a block's 32 products sum exactly in fp32, and scaling by a power of two is exact;
what rounds is the fp32 accumulation of K / 32 scaled block sums (relative 2^-24 each, against sum |block|) and the one
rounding of C to bf16: E1 <= 2e-2 as for every bf16 result, and, where all scales are equal (the sums are then the
unscaled ones times a power of two, exact in fp32), equality with the bf16 rounding of the oracle's value.
8-bit elements: the products are exact, a block's sum is not (36 binades of products against 24 bits), so only E1.
6-bit elements (a dense stream of codes, four to three bytes): E2M3 products span 12 binades with 8 significant bits, a
block's sum is exact in 24 bits and equal scales give equality as for E2M1; E3M2 products span 18 binades (2^-8 .. 784),
more than a 24-bit sum holds next to its largest term, so there only E1.
"""
import numpy as np
import pytest
import torch

import oracle
from inputs import synth
from paper_2602_12305_amd import binding as ob
from helpers import e1

pytestmark = pytest.mark.gpu
F4, F8, BF8, F6, BF6 = synth.DTYPE_F4E2M1, synth.DTYPE_F8E4M3, synth.DTYPE_F8E5M2, synth.DTYPE_F6E2M3, synth.DTYPE_F6E3M2
EIGHT = pytest.mark.parametrize("dt", [F8, BF8], ids=["e4m3", "e5m2"])
SIX = pytest.mark.parametrize("dt", [F6, BF6], ids=["e2m3", "e3m2"])


def quantised(seed, tag, rows, K, spread, dt=F4):
    """Rows of N(0, 1) values whose 32-blocks have magnitudes spread over 2^+-spread, quantised block by block."""
    x = synth.normal(seed, tag, rows, K)
    if spread:
        e = synth.integers(seed + 1, tag + "e", rows, K // 32, -spread, spread)
        x = x * np.repeat(np.exp2(e), 32, axis=1).astype(np.float32)
    codes, scales = synth.mx_quantize(x, dt)
    return np.ascontiguousarray(codes), np.ascontiguousarray(scales, dtype=np.uint8)          # codes come packed two to a byte


def run(As, sA, Bs, sB, bias, M, N, K, act, *, pad_c=0, pitch=0, spitch=0, shift=0, sshift=0, dt=F4):
    """pitch / spitch: extra bytes per row of the operands / of the scales; shift: bytes in front of every array;
    sshift: more bytes in front of the scale arrays only."""
    def dev(x, extra, front):
        rows, w = x.shape
        buf = np.full(front + rows * (w + extra), 0x5a, dtype=np.uint8)
        buf[front:].reshape(rows, w + extra)[:, :w] = x
        return torch.from_numpy(buf).cuda()[front - shift:], w + extra
    Ad, la = dev(As, pitch, shift); Bd, lb = dev(Bs, pitch, shift)
    sAd, lsa = dev(sA, spitch, shift + sshift); sBd, lsb = dev(sB, spitch, shift + sshift)
    bd = None if bias is None else torch.from_numpy(np.ascontiguousarray(bias, dtype=np.float32)).cuda()
    ldc = N + pad_c
    Cd = torch.full((M, ldc), 0x4442, dtype=torch.int16, device="cuda")
    num, den = (2, 1) if dt == F4 else (4, 3) if dt in (F6, BF6) else (1, 1)      # elements per stored byte
    args = (M, N, K, Ad[shift:], la * num // den, sAd[shift:], lsa, Bd[shift:], lb * num // den, sBd[shift:], lsb, bd, Cd, ldc)
    path = ob.optiml_gemm_epilogue_mx_path(*args, dt)
    ob.optiml_gemm_epilogue_mx(*args, dt, act)
    torch.cuda.synchronize()
    raw = Cd.cpu().numpy()
    assert np.all(raw[:, N:] == 0x4442)
    return synth.bf16_bits_to_f32(raw[:, :N].view(np.uint16)).astype(np.float64), path, raw


@pytest.mark.parametrize("M,N,K,want_path", [(256, 256, 512, 0), (300, 520, 1024, 0), (1024, 1000, 2048, 0), (512, 264, 384, 1), (512, 264, 640, 0),
                                             (300, 520, 480, 1), (100, 130, 256, 1), (17, 33, 32, 1), (260, 260, 96, 1)])
def test_block_scaled_contraction_matches_the_oracle(M, N, K, want_path):
    As, sA = quantised(7000 + M + K, "A", M, K, 6); Bs, sB = quantised(7000 + M + K, "B", N, K, 6)
    bias = synth.normal(7000 + M + K, "bias", 1, N)[0]
    for act in (synth.ACT_NONE, synth.ACT_SILU):
        got, path, raw = run(As, sA, Bs, sB, bias, M, N, K, act, pad_c=8)
        assert path == want_path
        ref = oracle.gemm_epilogue_mx(As, sA, Bs, sB, bias, M, N, K, dtype=F4, act=act)
        assert np.all(np.isfinite(got)) and e1(got, ref) <= 2e-2
        assert np.array_equal(run(As, sA, Bs, sB, bias, M, N, K, act, pad_c=8)[2], raw)          # bitwise repeatable
    got, path, _ = run(As, sA, Bs, sB, None, M, N, K, synth.ACT_RELU)
    assert e1(got, oracle.gemm_epilogue_mx(As, sA, Bs, sB, None, M, N, K, dtype=F4, act=synth.ACT_RELU)) <= 2e-2


def test_equal_scales_are_exact_and_every_scale_byte_lands_on_its_block():
    M, N, K = 300, 520, 1024
    As, _ = quantised(7100, "A", M, K, 0); Bs, _ = quantised(7100, "B", N, K, 0)
    for ea, eb in ((127, 127), (130, 121), (100, 140)):
        sA = np.full((M, K // 32), ea, dtype=np.uint8); sB = np.full((N, K // 32), eb, dtype=np.uint8)
        got, path, _ = run(As, sA, Bs, sB, None, M, N, K, synth.ACT_NONE)
        ref = oracle.gemm_epilogue_mx(As, sA, Bs, sB, None, M, N, K, dtype=F4, act=synth.ACT_NONE)
        assert path == 0 and np.array_equal(got, synth.bf16_bits_to_f32(oracle.bf16_from_double(ref)).astype(np.float64))
    # one block of one row of A scaled by 2^20, everything else by 2^0: only that row changes, by that block's share
    sA = np.full((M, K // 32), 127, dtype=np.uint8); sB = np.full((N, K // 32), 127, dtype=np.uint8)
    base, _, _ = run(As, sA, Bs, sB, None, M, N, K, synth.ACT_NONE)
    for row, blk in ((0, 0), (129, 5), (299, 31), (255, 17)):
        s2 = sA.copy(); s2[row, blk] = 147
        got, _, _ = run(As, s2, Bs, sB, None, M, N, K, synth.ACT_NONE)
        ref = oracle.gemm_epilogue_mx(As, s2, Bs, sB, None, M, N, K, dtype=F4, act=synth.ACT_NONE)
        assert e1(got, ref) <= 2e-2
        others = np.delete(np.arange(M), row)
        assert np.array_equal(got[others], base[others])
    for col, blk in ((0, 1), (519, 30), (256, 9)):                               # and of one column of B
        s2 = sB.copy(); s2[col, blk] = 147
        got, _, _ = run(As, sA, Bs, s2, None, M, N, K, synth.ACT_NONE)
        ref = oracle.gemm_epilogue_mx(As, sA, Bs, s2, None, M, N, K, dtype=F4, act=synth.ACT_NONE)
        assert e1(got, ref) <= 2e-2
        others = np.delete(np.arange(N), col)
        assert np.array_equal(got[:, others], base[:, others])


def test_pitches_offsets_and_degenerate_shapes():
    M, N, K = 264, 304, 640
    As, sA = quantised(7200, "A", M, K, 4); Bs, sB = quantised(7200, "B", N, K, 4)
    bias = synth.normal(7200, "bias", 1, N)[0]
    ref = oracle.gemm_epilogue_mx(As, sA, Bs, sB, bias, M, N, K, dtype=F4, act=synth.ACT_NONE)
    # the tile kernel takes any address and pitch of the scales (they are copied k-tile by k-tile first), but only
    # operands whose rows start on 16 bytes
    for kw, want in ((dict(pitch=16, spitch=4), 0), (dict(pitch=16, spitch=4, shift=16), 0), (dict(pitch=2, spitch=1), 1),
                     (dict(shift=3), 1), (dict(pitch=16, spitch=3), 0), (dict(sshift=1), 0), (dict(spitch=5, sshift=2), 0)):
        got, path, _ = run(As, sA, Bs, sB, bias, M, N, K, synth.ACT_NONE, **kw)
        assert path == want and e1(got, ref) <= 2e-2, kw
    # K = 0: act(bias); nothing to do for an empty C
    got, _, _ = run(As[:, :0], sA[:, :0], Bs[:, :0], sB[:, :0], bias, M, N, 0, synth.ACT_RELU)
    assert np.array_equal(got, np.broadcast_to(synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(np.maximum(bias, 0))).astype(np.float64), (M, N)))
    ob.optiml_gemm_epilogue_mx(0, 8, 32, None, 32, None, 1, None, 32, None, 1, None, None, 8, F4, 0)


def test_benchmark_size_on_sampled_rows_and_columns():
    M = N = K = 8192
    As, sA = quantised(7300, "A", M, K, 3); Bs, sB = quantised(7300, "B", N, K, 3)
    bias = synth.normal(7300, "bias", 1, N)[0]
    got, path, _ = run(As, sA, Bs, sB, bias, M, N, K, synth.ACT_SILU)
    assert path == 0
    rows = np.array([0, 1, 255, 256, 4097, 8190, 8191]); cols = np.array([0, 31, 32, 63, 64, 300, 4096, 8190, 8191])
    ref = oracle.gemm_epilogue_mx(np.ascontiguousarray(As[rows]), np.ascontiguousarray(sA[rows]), np.ascontiguousarray(Bs[cols]),
                                  np.ascontiguousarray(sB[cols]), bias[cols], len(rows), len(cols), K, dtype=F4, act=synth.ACT_SILU)
    assert e1(got[np.ix_(rows, cols)], ref) <= 2e-2


# ---- 8-bit elements (E4M3, E5M2): the 64-deep kernel, a k-tile of two blocks --------------------------------------

@EIGHT
@pytest.mark.parametrize("M,N,K,want_path", [(256, 256, 512, 0), (300, 520, 1024, 0), (1024, 1000, 2048, 0), (512, 264, 320, 0), (512, 264, 192, 1),
                                             (300, 520, 480, 1), (100, 130, 256, 1), (17, 33, 32, 1)])
def test_block_scaled_8bit_contraction_matches_the_oracle(M, N, K, want_path, dt):
    As, sA = quantised(7400 + M + K, "A", M, K, 6, dt); Bs, sB = quantised(7400 + M + K, "B", N, K, 6, dt)
    bias = synth.normal(7400 + M + K, "bias", 1, N)[0]
    for act in (synth.ACT_NONE, synth.ACT_SILU):
        got, path, raw = run(As, sA, Bs, sB, bias, M, N, K, act, pad_c=8, dt=dt)
        assert path == want_path
        ref = oracle.gemm_epilogue_mx(As, sA, Bs, sB, bias, M, N, K, dtype=dt, act=act)
        assert np.all(np.isfinite(got)) and e1(got, ref) <= 2e-2
        assert np.array_equal(run(As, sA, Bs, sB, bias, M, N, K, act, pad_c=8, dt=dt)[2], raw)      # bitwise repeatable


@EIGHT
def test_every_8bit_scale_byte_lands_on_its_block(dt):
    """One-hot rows of A pick single k positions, so a fragment byte fed to the wrong k slot or block cannot hide; then
    one block of one row (column) scaled by 2^20 changes exactly that row (column), by that block's share."""
    M, N, K = 300, 520, 1024
    A1 = np.zeros((M, K), dtype=np.float32); A1[np.arange(M), (37 * np.arange(M) + 11) % K] = 2.0
    As = synth.to_bits(A1, dt); Bs = synth.to_bits(synth.integers(7500, "B", N, K, -4, 4), dt)
    sA = (120 + synth.integers(7501, "sa", M, K // 32, 0, 14)).astype(np.uint8); sB = (120 + synth.integers(7502, "sb", N, K // 32, 0, 14)).astype(np.uint8)
    got, path, _ = run(As, sA, Bs, sB, None, M, N, K, synth.ACT_NONE, dt=dt)
    ref = oracle.gemm_epilogue_mx(As, sA, Bs, sB, None, M, N, K, dtype=dt, act=synth.ACT_NONE)
    assert path == 0 and np.array_equal(got, synth.bf16_bits_to_f32(oracle.bf16_from_double(ref)).astype(np.float64))   # one product per entry: exact
    As, _ = quantised(7510, "A", M, K, 0, dt); Bs, _ = quantised(7510, "B", N, K, 0, dt)
    sA = np.full((M, K // 32), 127, dtype=np.uint8); sB = np.full((N, K // 32), 127, dtype=np.uint8)
    base, _, _ = run(As, sA, Bs, sB, None, M, N, K, synth.ACT_NONE, dt=dt)
    for row, blk in ((0, 0), (129, 5), (299, 31), (255, 16)):
        s2 = sA.copy(); s2[row, blk] = 147
        got, _, _ = run(As, s2, Bs, sB, None, M, N, K, synth.ACT_NONE, dt=dt)
        assert e1(got, oracle.gemm_epilogue_mx(As, s2, Bs, sB, None, M, N, K, dtype=dt, act=synth.ACT_NONE)) <= 2e-2
        others = np.delete(np.arange(M), row)
        assert np.array_equal(got[others], base[others]) and not np.array_equal(got[row], base[row])
    for col, blk in ((0, 1), (519, 30), (256, 9)):
        s2 = sB.copy(); s2[col, blk] = 147
        got, _, _ = run(As, sA, Bs, s2, None, M, N, K, synth.ACT_NONE, dt=dt)
        assert e1(got, oracle.gemm_epilogue_mx(As, sA, Bs, s2, None, M, N, K, dtype=dt, act=synth.ACT_NONE)) <= 2e-2
        others = np.delete(np.arange(N), col)
        assert np.array_equal(got[:, others], base[:, others])


@EIGHT
def test_8bit_pitches_offsets_and_the_benchmark_size(dt):
    M, N, K = 264, 304, 640
    As, sA = quantised(7600, "A", M, K, 4, dt); Bs, sB = quantised(7600, "B", N, K, 4, dt)
    bias = synth.normal(7600, "bias", 1, N)[0]
    ref = oracle.gemm_epilogue_mx(As, sA, Bs, sB, bias, M, N, K, dtype=dt, act=synth.ACT_NONE)
    for kw, want in ((dict(pitch=16, spitch=2), 0), (dict(pitch=16, spitch=4, shift=16), 0), (dict(pitch=3, spitch=1), 1), (dict(shift=3), 1),
                     (dict(pitch=16, spitch=3, sshift=1), 0)):
        got, path, _ = run(As, sA, Bs, sB, bias, M, N, K, synth.ACT_NONE, dt=dt, **kw)
        assert path == want and e1(got, ref) <= 2e-2, kw
    M = N = K = 8192
    As, sA = quantised(7700, "A", M, K, 3, dt); Bs, sB = quantised(7700, "B", N, K, 3, dt)
    bias = synth.normal(7700, "bias", 1, N)[0]
    got, path, _ = run(As, sA, Bs, sB, bias, M, N, K, synth.ACT_SILU, dt=dt)
    assert path == 0
    rows = np.array([0, 1, 255, 256, 4097, 8190, 8191]); cols = np.array([0, 31, 32, 63, 64, 300, 4096, 8190, 8191])
    ref = oracle.gemm_epilogue_mx(np.ascontiguousarray(As[rows]), np.ascontiguousarray(sA[rows]), np.ascontiguousarray(Bs[cols]),
                                  np.ascontiguousarray(sB[cols]), bias[cols], len(rows), len(cols), K, dtype=dt, act=synth.ACT_SILU)
    assert e1(got[np.ix_(rows, cols)], ref) <= 2e-2


@SIX
@pytest.mark.parametrize("M,N,K,want_path", [(256, 256, 512, 0), (300, 520, 1024, 0), (1024, 1000, 2048, 0), (512, 264, 320, 0), (512, 264, 256, 0),
                                             (512, 264, 192, 1), (300, 520, 480, 1), (100, 130, 256, 1), (17, 33, 32, 1)])
def test_block_scaled_6bit_contraction_matches_the_oracle(M, N, K, want_path, dt):
    As, sA = quantised(7800 + M + K, "A", M, K, 6, dt); Bs, sB = quantised(7800 + M + K, "B", N, K, 6, dt)
    assert As.shape == (M, K * 3 // 4)
    bias = synth.normal(7800 + M + K, "bias", 1, N)[0]
    for act in (synth.ACT_NONE, synth.ACT_SILU):
        got, path, raw = run(As, sA, Bs, sB, bias, M, N, K, act, pad_c=8, dt=dt)
        assert path == want_path
        ref = oracle.gemm_epilogue_mx(As, sA, Bs, sB, bias, M, N, K, dtype=dt, act=act)
        assert np.all(np.isfinite(got)) and e1(got, ref) <= 2e-2
        assert np.array_equal(run(As, sA, Bs, sB, bias, M, N, K, act, pad_c=8, dt=dt)[2], raw)      # bitwise repeatable


@SIX
def test_every_6bit_scale_byte_lands_on_its_block(dt):
    """One-hot rows of A pick single k positions, so a code fed to the wrong k slot or block cannot hide; equal scales
    give the exact result; then one block of one row (column) scaled by 2^20 changes exactly that row (column)."""
    M, N, K = 300, 520, 1024
    A1 = np.zeros((M, K), dtype=np.float32); A1[np.arange(M), (37 * np.arange(M) + 11) % K] = 2.0
    As = synth.to_bits(A1, dt); Bs = synth.to_bits(synth.integers(7900, "B", N, K, -4, 4), dt)
    sA = (120 + synth.integers(7901, "sa", M, K // 32, 0, 14)).astype(np.uint8); sB = (120 + synth.integers(7902, "sb", N, K // 32, 0, 14)).astype(np.uint8)
    got, path, _ = run(As, sA, Bs, sB, None, M, N, K, synth.ACT_NONE, dt=dt)
    ref = oracle.gemm_epilogue_mx(As, sA, Bs, sB, None, M, N, K, dtype=dt, act=synth.ACT_NONE)
    assert path == 0 and np.array_equal(got, synth.bf16_bits_to_f32(oracle.bf16_from_double(ref)).astype(np.float64))   # one product per entry: exact
    As, _ = quantised(7910, "A", M, K, 0, dt); Bs, _ = quantised(7910, "B", N, K, 0, dt)
    sA = np.full((M, K // 32), 127, dtype=np.uint8); sB = np.full((N, K // 32), 125, dtype=np.uint8)
    base, _, _ = run(As, sA, Bs, sB, None, M, N, K, synth.ACT_NONE, dt=dt)
    ref = oracle.gemm_epilogue_mx(As, sA, Bs, sB, None, M, N, K, dtype=dt, act=synth.ACT_NONE)
    if dt == F6:
        assert np.array_equal(base, synth.bf16_bits_to_f32(oracle.bf16_from_double(ref)).astype(np.float64))            # equal scales: exact
    else:
        assert e1(base, ref) <= 2e-2
    for row, blk in ((0, 0), (129, 5), (299, 31), (255, 16)):
        s2 = sA.copy(); s2[row, blk] = 147
        got, _, _ = run(As, s2, Bs, sB, None, M, N, K, synth.ACT_NONE, dt=dt)
        assert e1(got, oracle.gemm_epilogue_mx(As, s2, Bs, sB, None, M, N, K, dtype=dt, act=synth.ACT_NONE)) <= 2e-2
        others = np.delete(np.arange(M), row)
        assert np.array_equal(got[others], base[others]) and not np.array_equal(got[row], base[row])
    for col, blk in ((0, 1), (519, 30), (256, 9)):
        s2 = sB.copy(); s2[col, blk] = 147
        got, _, _ = run(As, sA, Bs, s2, None, M, N, K, synth.ACT_NONE, dt=dt)
        assert e1(got, oracle.gemm_epilogue_mx(As, sA, Bs, s2, None, M, N, K, dtype=dt, act=synth.ACT_NONE)) <= 2e-2
        others = np.delete(np.arange(N), col)
        assert np.array_equal(got[:, others], base[:, others])


@SIX
def test_6bit_pitches_offsets_and_the_benchmark_size(dt):
    M, N, K = 264, 304, 640
    As, sA = quantised(8000, "A", M, K, 4, dt); Bs, sB = quantised(8000, "B", N, K, 4, dt)
    bias = synth.normal(8000, "bias", 1, N)[0]
    ref = oracle.gemm_epilogue_mx(As, sA, Bs, sB, bias, M, N, K, dtype=dt, act=synth.ACT_NONE)
    # the operands are copied: any pitch that keeps rows on bytes (extra bytes a multiple of 3), any address
    for kw in (dict(pitch=48, spitch=2), dict(pitch=48, spitch=4, shift=16), dict(pitch=3, spitch=1), dict(shift=3), dict(pitch=6, spitch=3, sshift=1)):
        got, path, _ = run(As, sA, Bs, sB, bias, M, N, K, synth.ACT_NONE, dt=dt, **kw)
        assert path == 0 and e1(got, ref) <= 2e-2, kw
    M = N = K = 8192
    As, sA = quantised(8100, "A", M, K, 3, dt); Bs, sB = quantised(8100, "B", N, K, 3, dt)
    bias = synth.normal(8100, "bias", 1, N)[0]
    got, path, _ = run(As, sA, Bs, sB, bias, M, N, K, synth.ACT_SILU, dt=dt)
    assert path == 0
    rows = np.array([0, 1, 255, 256, 4097, 8190, 8191]); cols = np.array([0, 31, 32, 63, 64, 300, 4096, 8190, 8191])
    ref = oracle.gemm_epilogue_mx(np.ascontiguousarray(As[rows]), np.ascontiguousarray(sA[rows]), np.ascontiguousarray(Bs[cols]),
                                  np.ascontiguousarray(sB[cols]), bias[cols], len(rows), len(cols), K, dtype=dt, act=synth.ACT_SILU)
    assert e1(got[np.ix_(rows, cols)], ref) <= 2e-2


@pytest.mark.parametrize("M,N,K", [(16, 2048, 1024), (5, 1030, 384), (128, 1024, 512), (40, 8200, 256), (1, 16384, 128), (17, 8192, 2048)])
def test_few_rows_of_block_scaled_e2m1_take_the_streaming_kernel(M, N, K):
    As, sA = quantised(8200 + M + K, "A", M, K, 6); Bs, sB = quantised(8200 + M + K, "B", N, K, 6)
    bias = synth.normal(8200 + M + K, "bias", 1, N)[0]
    for act in (synth.ACT_NONE, synth.ACT_SILU):
        got, path, raw = run(As, sA, Bs, sB, bias, M, N, K, act, pad_c=8)
        assert path == 2
        ref = oracle.gemm_epilogue_mx(As, sA, Bs, sB, bias, M, N, K, dtype=F4, act=act)
        assert np.all(np.isfinite(got)) and e1(got, ref) <= 2e-2
        assert np.array_equal(run(As, sA, Bs, sB, bias, M, N, K, act, pad_c=8)[2], raw)          # bitwise repeatable
    # equal scales: exact; pitches and offsets that keep the rows on 16-byte boundaries, any scale address
    one = np.full_like(sA, 125); oneB = np.full_like(sB, 130)
    got, path, _ = run(As, one, Bs, oneB, None, M, N, K, synth.ACT_NONE, pitch=16, spitch=3, shift=16, sshift=1)
    ref = oracle.gemm_epilogue_mx(As, one, Bs, oneB, None, M, N, K, dtype=F4, act=synth.ACT_NONE)
    assert path == 2 and np.array_equal(got, synth.bf16_bits_to_f32(oracle.bf16_from_double(ref)).astype(np.float64))
    # rows off the 16-byte grid go elsewhere
    assert run(As, sA, Bs, sB, bias, M, N, K, synth.ACT_NONE, shift=3)[1] != 2


def test_every_scale_byte_lands_on_its_block_in_the_streaming_kernel():
    """One-hot rows of A pick single k positions; then one block of one row (column) scaled by 2^20 changes exactly that
    row (column)."""
    M, N, K = 16, 1040, 1024
    A1 = np.zeros((M, K), dtype=np.float32); A1[np.arange(M), (37 * np.arange(M) + 11) % K] = 2.0
    As = synth.to_bits(A1, F4); Bs = synth.to_bits(synth.integers(8300, "B", N, K, -4, 4), F4)
    sA = (120 + synth.integers(8301, "sa", M, K // 32, 0, 14)).astype(np.uint8); sB = (120 + synth.integers(8302, "sb", N, K // 32, 0, 14)).astype(np.uint8)
    got, path, _ = run(As, sA, Bs, sB, None, M, N, K, synth.ACT_NONE)
    ref = oracle.gemm_epilogue_mx(As, sA, Bs, sB, None, M, N, K, dtype=F4, act=synth.ACT_NONE)
    assert path == 2 and np.array_equal(got, synth.bf16_bits_to_f32(oracle.bf16_from_double(ref)).astype(np.float64))   # one product per entry: exact
    As, _ = quantised(8310, "A", M, K, 0); Bs, _ = quantised(8310, "B", N, K, 0)
    sA = np.full((M, K // 32), 127, dtype=np.uint8); sB = np.full((N, K // 32), 127, dtype=np.uint8)
    base, _, _ = run(As, sA, Bs, sB, None, M, N, K, synth.ACT_NONE)
    for row, blk in ((0, 0), (9, 5), (15, 31)):
        s2 = sA.copy(); s2[row, blk] = 147
        got, _, _ = run(As, s2, Bs, sB, None, M, N, K, synth.ACT_NONE)
        assert e1(got, oracle.gemm_epilogue_mx(As, s2, Bs, sB, None, M, N, K, dtype=F4, act=synth.ACT_NONE)) <= 2e-2
        others = np.delete(np.arange(M), row)
        assert np.array_equal(got[others], base[others]) and not np.array_equal(got[row], base[row])
    for col, blk in ((0, 1), (1039, 30), (256, 9)):
        s2 = sB.copy(); s2[col, blk] = 147
        got, _, _ = run(As, sA, Bs, s2, None, M, N, K, synth.ACT_NONE)
        assert e1(got, oracle.gemm_epilogue_mx(As, sA, Bs, s2, None, M, N, K, dtype=F4, act=synth.ACT_NONE)) <= 2e-2
        others = np.delete(np.arange(N), col)
        assert np.array_equal(got[:, others], base[:, others])
    # a NaN scale poisons exactly its row
    s2 = sA.copy(); s2[3, 7] = 255
    got, _, _ = run(As, s2, Bs, sB, None, M, N, K, synth.ACT_NONE)
    assert np.all(np.isnan(got[3])) and not np.any(np.isnan(np.delete(got, 3, 0)))
