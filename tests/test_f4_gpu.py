"""4-bit E2M1 operands (two to a byte along k, no scale factors) against the CPU oracle, element by element.

Every E2M1 value is a multiple of 0.5 of magnitude at most 6, so every product is a multiple of 0.25 of magnitude at most
36 and a sum of K <= 16384 of them is exact in fp32 in any order: with a bias of multiples of 0.25 and no activation
(or ReLU) the kernels must return exactly the bf16 rounding of the oracle's value.  With SiLU / GELU the bar is the
bf16 contraction's, E1 <= 2e-2.
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
F4 = synth.DTYPE_F4E2M1


def chosen(M, N, K, layout=1, batch=1):
    P = 0x10000
    v = ob.optiml_select_variant(batch, M, N, K, P, K, M * K, P, K, K * N, P, N, P, M if layout & 4 else N, M * N, layout, F4, 0)
    return ob.optiml_variant_name(v)


def operands(seed, M, N, K, batch=None, scale=2.0):
    A = synth.normal(seed, "A", M, K, batch=batch) * np.float32(scale)
    B = synth.normal(seed, "B", K, N, batch=batch) * np.float32(scale)
    bias = np.round(synth.normal(seed, "bias", 1, N)[0] * 8.0) / 4.0            # multiples of 0.25
    return A, B, bias.astype(np.float32)


@pytest.mark.parametrize("M,N,K,family", [(300, 520, 1024, "skinnyrc_f4"), (16, 2048, 4096, "skinnyrc_f4"), (5, 1000, 2048, "skinnyrc_f4"),
                                          (100, 130, 70, "generic"), (33, 65, 2, "generic")])
def test_dispatched_kernels_are_exact_and_match_the_oracle(M, N, K, family):
    assert chosen(M, N, K).startswith(family)
    A, B, bias = operands(5000 + M + K, M, N, K)
    for act in (synth.ACT_NONE, synth.ACT_RELU):
        check_against_oracle(A, B, bias, dtype=F4, act=act, layout=1, exact=True)
    check_against_oracle(A, B, None, dtype=F4, act=synth.ACT_NONE, layout=1, exact=True, ldc_pad=8)
    for act in (synth.ACT_SILU, synth.ACT_GELU_TANH):
        check_against_oracle(A * np.float32(0.25), B * np.float32(0.25), bias, dtype=F4, act=act, layout=1)


def sampled_check(M, N, K, seed, act, exact):
    """Whole problem on the GPU; the oracle on sampled rows and columns (tile edges, the ragged ends, a spread)."""
    A = synth.f32_to_f4e2m1_codes(synth.normal(seed, "A", M, K) * np.float32(2.0))
    B = synth.f32_to_f4e2m1_codes(synth.normal(seed, "B", N, K) * np.float32(2.0))      # stored [N][K]
    bias = (np.round(synth.normal(seed, "bias", 1, N)[0] * 8.0) / 4.0).astype(np.float32)
    As, Bs = synth.pack_f4(A), synth.pack_f4(B)
    Y, _, _ = run_gpu(As, Bs, bias, 1, M, N, K, F4, act, 1)
    rows = np.unique(np.clip(np.concatenate([[0, 1, 127, 128, 255, 256, 257, M // 2, M - 2, M - 1], np.arange(13, M, max(1, M // 7))]), 0, M - 1))
    cols = np.unique(np.clip(np.concatenate([[0, 31, 32, 63, 64, 255, 256, N // 2, N - 2, N - 1], np.arange(5, N, max(1, N // 9))]), 0, N - 1))
    ref = oracle.gemm_epilogue(np.ascontiguousarray(As[rows]), np.ascontiguousarray(Bs[cols]), bias[cols], len(rows), len(cols), K,
                               dtype=F4, act=act, layout=1)[0]
    got = Y[0][np.ix_(rows, cols)]
    if exact:
        assert np.array_equal(got, synth.bf16_bits_to_f32(oracle.bf16_from_double(ref)).astype(np.float64))
    else:
        assert e1(got, ref) <= 2e-2


@pytest.mark.parametrize("M,N,K,family", [(2048, 2048, 2048, "ring_f4_rc"), (3000, 3000, 3008, "ring_f4_rc"), (2000, 2056, 2080, "ring_f4_rc"),
                                          (1300, 2300, 6144, "xpad"), (48, 4096, 8192, "skinnyrc_f4"), (1024, 1024, 4096, "skinnyrc_f4")])
def test_larger_dispatched_problems_on_sampled_entries(M, N, K, family):
    assert chosen(M, N, K).startswith(family)
    sampled_check(M, N, K, 5300 + M, synth.ACT_NONE, True)
    sampled_check(M, N, K, 5400 + M, synth.ACT_SILU, False)


def test_every_code_pair_multiplies_exactly():
    # all 16 x 16 pairs of codes, one pair per (row, column), K = 2: C[i][j] = value(i) * value(j) + 0 * 0
    codes = np.arange(16, dtype=np.uint8)
    vals = synth.f4e2m1_codes_to_f32(codes)
    As = np.stack([codes, np.zeros(16, np.uint8)], axis=1)                      # rows of 2 elements: (code, +0)
    packed = synth.pack_f4(As)
    Y, _, _ = run_gpu(packed, packed, None, 1, 16, 16, 2, F4, synth.ACT_NONE, 1)
    want = np.outer(vals, vals).astype(np.float64)
    assert np.array_equal(Y[0], want)
    # the odd element of a byte is the high half
    packed_hi = synth.pack_f4(np.stack([np.zeros(16, np.uint8), codes], axis=1))
    Y2, _, _ = run_gpu(packed_hi, packed, None, 1, 16, 16, 2, F4, synth.ACT_NONE, 1)
    assert np.all(Y2[0] == 0.0)                                                  # high halves of A meet the +0 of B
    Y3, _, _ = run_gpu(packed_hi, packed_hi, None, 1, 16, 16, 2, F4, synth.ACT_NONE, 1)
    assert np.array_equal(Y3[0], want)


def test_column_major_c_batches_pitches_and_repeatability():
    M, N, K, batch = 260, 392, 1024, 3
    A, B, _ = operands(5100, M, N, K, batch=batch)
    bias = (np.round(synth.normal(5100, "bias", 1, N, batch=batch).reshape(batch, N) * 8.0) / 4.0).astype(np.float32)
    As, Bs = store(A, F4, False, 32), store(B, F4, True, 64)                     # pitches beyond the rows
    Y1, _, C1 = run_gpu(As, Bs, bias, batch, M, N, K, F4, synth.ACT_NONE, 1)
    Y2, _, C2 = run_gpu(As, Bs, bias, batch, M, N, K, F4, synth.ACT_NONE, 1)
    assert torch.equal(C1, C2)
    ref = oracle.gemm_epilogue(As, Bs, bias, M, N, K, dtype=F4, act=synth.ACT_NONE, layout=1, batch=batch)
    want = synth.bf16_bits_to_f32(oracle.bf16_from_double(ref)).astype(np.float64)
    assert np.array_equal(Y1, want)
    # column-major C: the mirror-image problem
    Yc, _, _ = run_gpu(As, Bs, None, batch, M, N, K, F4, synth.ACT_RELU, 5)
    refc = oracle.gemm_epilogue(As, Bs, None, M, N, K, dtype=F4, act=synth.ACT_RELU, layout=1, batch=batch)
    assert np.array_equal(Yc, synth.bf16_bits_to_f32(oracle.bf16_from_double(refc)).astype(np.float64))


def test_benchmark_size_on_sampled_entries():
    """8192^3 as the benchmark times it: sampled rows and columns against the oracle, exactly."""
    assert chosen(8192, 8192, 8192).startswith("ring_f4_rc_256x256")
    sampled_check(8192, 8192, 8192, 5200, synth.ACT_NONE, True)
