"""6-bit E2M3 and E3M2 operands (a dense little-endian stream of 6-bit codes, no scale factors) against the CPU oracle,
element by element.

E2M3 values are multiples of 1/8 of magnitude at most 7.5, E3M2 values multiples of 1/16 of magnitude at most 28: every
product is a multiple of 2^-8 below 2^10, and on the N(0, 4)-distributed operands used here every partial sum of up to
8192 of them stays far below 2^16, so all sums are exact in fp32 in any order: with a bias of multiples of 0.25 and no
activation (or ReLU) the kernels must return exactly the bf16 rounding of the oracle's value.  With SiLU / GELU the bar
is the bf16 contraction's, E1 <= 2e-2.
"""
import numpy as np
import pytest
import torch

import oracle
from inputs import synth
from paper_2602_12305_amd import binding as ob
from gpu_harness import check_against_oracle, run_gpu
from helpers import e1, store

pytestmark = pytest.mark.gpu
F6, BF6 = synth.DTYPE_F6E2M3, synth.DTYPE_F6E3M2
BOTH = pytest.mark.parametrize("dt", [F6, BF6], ids=["e2m3", "e3m2"])
TAG = {F6: "f6", BF6: "bf6"}


def chosen(dt, M, N, K, layout=1, batch=1):
    P = 0x10000
    a_ld, b_ld = (M if layout & 2 else K), (K if layout & 1 else N)
    v = ob.optiml_select_variant(batch, M, N, K, P, a_ld, M * K, P, b_ld, K * N, P, N, P, M if layout & 4 else N, M * N, layout, dt, 0)
    return ob.optiml_variant_name(v)


def operands(seed, M, N, K, batch=None, scale=2.0):
    A = synth.normal(seed, "A", M, K, batch=batch) * np.float32(scale)
    B = synth.normal(seed, "B", K, N, batch=batch) * np.float32(scale)
    bias = np.round(synth.normal(seed, "bias", 1, N)[0] * 8.0) / 4.0            # multiples of 0.25
    return A, B, bias.astype(np.float32)


@BOTH
@pytest.mark.parametrize("M,N,K,family", [(300, 520, 1024, "xs_ring"), (5, 1000, 2048, "stream6"), (16, 4100, 4128, "stream6"), (1, 17, 32, "stream6"), (16, 1030, 4224, "stream6"),
                                          (3, 16400, 1152, "stream6"), (40, 1000, 2048, "stream6"), (128, 520, 1056, "stream6"), (17, 4096, 4096, "stream6"),
                                          (5, 1000, 2052, "xs_ring"), (129, 264, 228, "xs_ring"),
                                          (64, 64, 512, "stream6"), (100, 130, 36, "generic"), (33, 65, 4, "generic"),
                                          (300, 520, 100, "generic")])
def test_dispatched_kernels_are_exact_and_match_the_oracle(dt, M, N, K, family):
    assert chosen(dt, M, N, K).startswith(family + ("_" + TAG[dt] if family != "generic" else ""))
    A, B, bias = operands(5600 + M + K, M, N, K)
    for act in (synth.ACT_NONE, synth.ACT_RELU):
        check_against_oracle(A, B, bias, dtype=dt, act=act, layout=1, exact=True)
    check_against_oracle(A, B, None, dtype=dt, act=synth.ACT_NONE, layout=1, exact=True, ldc_pad=8)
    for act in (synth.ACT_SILU, synth.ACT_GELU_TANH):
        check_against_oracle(A * np.float32(0.25), B * np.float32(0.25), bias, dtype=dt, act=act, layout=1)


@BOTH
@pytest.mark.parametrize("layout", [0, 2, 3])
def test_other_layouts_take_the_fallback_and_match_the_oracle(dt, layout):
    M, N, K = 68, 132, 40
    assert chosen(dt, M, N, K, layout=layout).startswith("generic")
    A, B, bias = operands(5700 + layout, M, N, K)
    check_against_oracle(A, B, bias, dtype=dt, act=synth.ACT_RELU, layout=layout, exact=True)


@BOTH
def test_every_code_pair_multiplies_exactly_at_every_position_of_the_stream(dt):
    # all 64 x 64 pairs of codes, one pair per (row, column); the pair sits at element p of a row of K, the rest is +0
    codes = np.arange(64, dtype=np.uint8)
    vals = synth.f6_codes_to_f32(codes, dt)
    want = np.outer(vals, vals).astype(np.float64)
    xs = ob.variant_names().index("xs_ring_" + TAG[dt] + "_rc_256x256_w2x4_ns5_k64")
    for K, positions in ((4, (0, 1, 2, 3)), (128, (0, 5, 31, 32, 63, 64, 95, 127)), (320, (21, 42, 170, 319))):
        # the dispatcher's kernel (the fallback for K = 4, a streaming kernel otherwise) and the copy into slots + ring kernel
        assert chosen(dt, 64, 64, K).startswith("stream6" if K >= 128 else "generic")
        for variant in (None, xs) if K >= 128 else (None,):
            for pos in positions:
                rows = np.zeros((64, K), dtype=np.uint8); rows[:, pos] = codes
                packed = synth.pack_f6(rows)
                Y, _, _ = run_gpu(packed, packed, None, 1, 64, 64, K, dt, synth.ACT_NONE, 1, variant=variant)
                assert np.array_equal(Y[0], want), (K, pos, variant)
                other = np.zeros((64, K), dtype=np.uint8); other[:, (pos + 1) % K] = codes
                Y2, _, _ = run_gpu(synth.pack_f6(other), packed, None, 1, 64, 64, K, dt, synth.ACT_NONE, 1, variant=variant)
                assert np.all(Y2[0] == 0.0), (K, pos, variant)                  # neighbouring positions do not meet


@BOTH
def test_column_major_c_batches_pitches_and_repeatability(dt):
    M, N, K, batch = 260, 392, 1000, 3
    A, B, _ = operands(5800, M, N, K, batch=batch)
    bias = (np.round(synth.normal(5800, "bias", 1, N, batch=batch).reshape(batch, N) * 8.0) / 4.0).astype(np.float32)
    As, Bs = store(A, dt, False, 24), store(B, dt, True, 88)                     # pitches beyond the rows: 768 and 816 bytes
    Y1, _, C1 = run_gpu(As, Bs, bias, batch, M, N, K, dt, synth.ACT_NONE, 1)
    Y2, _, C2 = run_gpu(As, Bs, bias, batch, M, N, K, dt, synth.ACT_NONE, 1)
    assert torch.equal(C1, C2)
    ref = oracle.gemm_epilogue(As, Bs, bias, M, N, K, dtype=dt, act=synth.ACT_NONE, layout=1, batch=batch)
    assert np.array_equal(Y1, synth.bf16_bits_to_f32(oracle.bf16_from_double(ref)).astype(np.float64))
    # rows that do not start on 16-byte boundaries (pitch 753 bytes): the copy's byte path
    As2, Bs2 = store(A, dt, False, 4), store(B, dt, True, 4)
    Y3, _, _ = run_gpu(As2, Bs2, bias, batch, M, N, K, dt, synth.ACT_NONE, 1)
    assert np.array_equal(Y3, Y1)
    # column-major C: the mirror-image problem
    Yc, _, _ = run_gpu(As, Bs, None, batch, M, N, K, dt, synth.ACT_RELU, 5)
    refc = oracle.gemm_epilogue(As, Bs, None, M, N, K, dtype=dt, act=synth.ACT_RELU, layout=1, batch=batch)
    assert np.array_equal(Yc, synth.bf16_bits_to_f32(oracle.bf16_from_double(refc)).astype(np.float64))


def sampled_check(dt, M, N, K, seed, act, exact):
    """Whole problem on the GPU; the oracle on sampled rows and columns (tile edges, the ragged ends, a spread)."""
    As = synth.pack_f6(synth.f32_to_f6_codes(synth.normal(seed, "A", M, K) * np.float32(2.0), dt))
    Bs = synth.pack_f6(synth.f32_to_f6_codes(synth.normal(seed, "B", N, K) * np.float32(2.0), dt))     # stored [N][K]
    bias = (np.round(synth.normal(seed, "bias", 1, N)[0] * 8.0) / 4.0).astype(np.float32)
    Y, _, _ = run_gpu(As, Bs, bias, 1, M, N, K, dt, act, 1)
    rows = np.unique(np.clip(np.concatenate([[0, 1, 127, 128, 255, 256, 257, M // 2, M - 2, M - 1], np.arange(13, M, max(1, M // 7))]), 0, M - 1))
    cols = np.unique(np.clip(np.concatenate([[0, 31, 32, 63, 64, 255, 256, N // 2, N - 2, N - 1], np.arange(5, N, max(1, N // 9))]), 0, N - 1))
    ref = oracle.gemm_epilogue(np.ascontiguousarray(As[rows]), np.ascontiguousarray(Bs[cols]), bias[cols], len(rows), len(cols), K,
                               dtype=dt, act=act, layout=1)[0]
    got = Y[0][np.ix_(rows, cols)]
    if exact:
        assert np.array_equal(got, synth.bf16_bits_to_f32(oracle.bf16_from_double(ref)).astype(np.float64))
    else:
        assert e1(got, ref) <= 2e-2


@BOTH
@pytest.mark.parametrize("M,N,K", [(2048, 2048, 2048), (3000, 3000, 3004), (2000, 2056, 2080)])
def test_larger_dispatched_problems_on_sampled_entries(dt, M, N, K):
    assert chosen(dt, M, N, K).startswith("xs_ring_" + TAG[dt])
    sampled_check(dt, M, N, K, 5900 + M, synth.ACT_NONE, True)
    sampled_check(dt, M, N, K, 6000 + M, synth.ACT_SILU, False)


@BOTH
def test_benchmark_size_on_sampled_entries(dt):
    """8192^3 as the benchmark times it: sampled rows and columns against the oracle, exactly."""
    assert chosen(dt, 8192, 8192, 8192).startswith("xs_ring_" + TAG[dt])
    sampled_check(dt, 8192, 8192, 8192, 6100, synth.ACT_NONE, True)


@BOTH
def test_degenerate_shapes(dt):
    """K = 0 gives act(bias); M = 0 or N = 0 writes nothing; a single row, a single column, K = 4 (one 3-byte group)."""
    N = 40
    bias = (np.arange(N, dtype=np.float32) - 20.0) / 4.0
    empty = np.zeros((8, 0), dtype=np.uint8)
    Y, _, _ = run_gpu(empty, np.zeros((N, 0), dtype=np.uint8), bias, 1, 8, N, 0, dt, synth.ACT_RELU, 1)
    assert np.array_equal(Y[0], np.tile(np.maximum(bias, 0.0).astype(np.float64), (8, 1)))
    P = torch.full((4, 64), 0x4442, dtype=torch.int16, device="cuda")
    A = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    ob.optiml_gemm_epilogue_ex(0, 64, 64, A, 64, A, 64, None, P, 64, 1, dt, 0)
    ob.optiml_gemm_epilogue_ex(4, 0, 64, A, 64, A, 64, None, P, 64, 1, dt, 0)
    torch.cuda.synchronize()
    assert bool((P == 0x4442).all())
    for M, Nn, K in ((1, 8, 4), (8, 1, 4), (1, 1, 1024), (3, 5, 68)):
        A, B, b = operands(6200 + M + K, M, Nn, K)
        check_against_oracle(A, B, b, dtype=dt, act=synth.ACT_NONE, layout=1, exact=True)


@BOTH
@pytest.mark.parametrize("M,N,K", [(1000, 24, 2048), (520, 100, 1056), (4100, 16, 4096)])
def test_few_columns_with_a_column_major_result(dt, M, N, K):
    """Column-major C is served as the mirror-image problem (C^T = B^T A^T, the bias running down its rows): with few
    columns that is a few-row problem for the streaming kernels, bias indexed by the row."""
    A, B, bias = operands(6300 + N + K, M, N, K)
    check_against_oracle(A, B, bias, dtype=dt, act=synth.ACT_RELU, layout=5, exact=True)
    check_against_oracle(A * np.float32(0.25), B * np.float32(0.25), bias, dtype=dt, act=synth.ACT_SILU, layout=5, ldc_pad=8)
