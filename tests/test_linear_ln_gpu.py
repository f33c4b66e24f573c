"""Parity of the contraction fused with LayerNorm over the rows of the product (paper Table 4, task 2 into task 4)
with the CPU oracle, element by element, through the C-ABI.

Bar.  y = (z - mu) / s with s = sqrt(var + eps).  The kernels accumulate products in fp32: every z is off by at most
d = 16 * 2^-24 * max_j (|bias_j| + sum_k |a_ik b_kj|) over the row (the componentwise bound the contraction's own
tests use).  Then |d mu| <= d, |d s| <= d (the root mean square is 1-Lipschitz in the maximum norm), so
|d y| <= (2 d + |y| d) / s.  The slice means and squared deviations are formed in fp32 from at most 64 values
(relative 2^-24 times a small constant) and merged in fp64: 2e-6 (1 + |y|) covers them; the result is rounded once
to the storage type: half a step of it (fp32 2^-24, bf16 2^-8, binary16 2^-11 relative, plus the subnormal floor).
"""
import numpy as np
import pytest
import torch

import oracle
from inputs import synth
from paper_2602_12305_amd import binding as ob
from gpu_harness import to_dev
from helpers import store

pytestmark = pytest.mark.gpu
F32, BF16, F16 = synth.DTYPE_F32, synth.DTYPE_BF16, synth.DTYPE_F16
HALF_STEP = {F32: 2.0 ** -24, BF16: 2.0 ** -8, F16: 2.0 ** -11}
FLOOR = {F32: 2.0 ** -149, BF16: 2.0 ** -133, F16: 2.0 ** -24}


def run(As, Bs, bias, M, N, K, layout, dtype, eps, pad=0, shift=0):
    """Y with `pad` extra elements per row and `shift` elements in front (poisoned); returns (values as fp64 [M, N], path)."""
    Ad, Bd = to_dev(As), to_dev(Bs)
    bd = None if bias is None else torch.from_numpy(np.ascontiguousarray(bias, dtype=np.float32)).cuda()
    ldy = N + pad
    tdt = torch.float32 if dtype == F32 else torch.int16
    poison = 777.0 if dtype == F32 else 0x4442
    buf = torch.full((shift + max(M, 1) * ldy,), poison, dtype=tdt, device="cuda")
    Y = buf[shift:]
    path = ob.optiml_gemm_layernorm_path(M, N, K, Ad, As.shape[-1], Bd, Bs.shape[-1], bd, Y, ldy, layout, dtype)
    ob.optiml_gemm_layernorm(M, N, K, Ad, As.shape[-1], Bd, Bs.shape[-1], bd, Y, ldy, eps, layout, dtype)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    body = host[shift:shift + M * ldy].reshape(M, ldy)
    assert np.all(host[:shift] == poison) and np.all(body[:, N:] == poison)          # padding untouched
    got = body[:, :N]
    if dtype != F32:
        got = synth.from_bits(np.ascontiguousarray(got).view(np.uint16), dtype)
    return got.astype(np.float64), path, body.copy()


def check(M, N, K, layout, dtype, seed, want_path, *, use_bias=True, pad=0, shift=0, scale=1.0, eps=1e-5, opad=0):
    A = synth.normal(seed, "A", M, K) * np.float32(scale); B = synth.normal(seed, "B", K, N)
    bias = (synth.normal(seed, "bias", 1, N)[0] * np.float32(3.0) + np.float32(1.5)) if use_bias else None
    As = store(A, dtype, (layout >> 1) & 1, opad); Bs = store(B, dtype, layout & 1, opad)
    got, path, raw = run(As, Bs, bias, M, N, K, layout, dtype, eps, pad, shift)
    assert path == want_path
    z, den = oracle.gemm_epilogue(As, Bs, bias, M, N, K, dtype=dtype, layout=layout, want_absden=True)
    z = z.reshape(M, N); den = den.reshape(M, N)
    ref = oracle.gemm_layernorm(As, Bs, bias, M, N, K, dtype=dtype, layout=layout, eps=eps)
    s = np.sqrt(z.var(axis=1, keepdims=True) + eps)
    d = 16 * 2.0 ** -24 * den.max(axis=1, keepdims=True)
    tol = d * (2.0 + np.abs(ref)) / s + 2e-6 * (1.0 + np.abs(ref)) + HALF_STEP[dtype] * np.abs(ref) + FLOOR[dtype]
    err = np.abs(got - ref)
    worst = np.unravel_index(int(np.argmax(err - tol)), err.shape)
    assert np.all(np.isfinite(got)) and np.all(err <= tol), (worst, got[worst], ref[worst], tol[worst])
    again = run(As, Bs, bias, M, N, K, layout, dtype, eps, pad, shift)[2]
    assert np.array_equal(again, raw)                                                # bitwise repeatable
    return got, ref


@pytest.mark.parametrize("dtype", [BF16, F16])
@pytest.mark.parametrize("layout,M,N,K", [(0, 300, 520, 160), (1, 300, 515, 160), (0, 1024, 4096, 512), (1, 77, 64, 128),
                                          (0, 513, 264, 992), (1, 256, 1000, 1024), (0, 300, 520, 344), (1, 300, 515, 376)])
def test_matrix_pipe_path_matches_the_oracle(dtype, layout, M, N, K):
    check(M, N, K, layout, dtype, 4000 + N, 0)
    check(M, N, K, layout, dtype, 4100 + N, 0, use_bias=False, scale=0.25, pad=3, shift=1)     # Y anywhere, any pitch


@pytest.mark.parametrize("layout,M,N,K", [(0, 300, 520, 160), (1, 300, 515, 160), (0, 1024, 2048, 512), (1, 77, 64, 64),
                                          (0, 513, 264, 1008), (1, 130, 1000, 2048), (0, 300, 520, 172), (1, 300, 515, 184)])
def test_fp32_matrix_pipe_path_matches_the_oracle(layout, M, N, K):
    check(M, N, K, layout, F32, 4500 + N, 0, pad=(-N) % 4)
    check(M, N, K, layout, F32, 4600 + N, 0, use_bias=False, scale=0.25, pad=(-N) % 4 + 4)      # a pitch that keeps rows aligned


@pytest.mark.parametrize("dtype,layout,M,N,K,opad,pad", [(F32, 0, 37, 53, 29, 0, 0), (F32, 1, 40, 300, 48, 4, 1), (F32, 2, 33, 257, 100, 0, 0),
                                                         (F32, 3, 5, 1000, 7, 1, 3), (BF16, 2, 64, 512, 128, 0, 0), (F16, 0, 50, 77, 45, 0, 5),
                                                         (BF16, 0, 20, 516, 160, 0, 0), (F32, 0, 3, 1, 16, 0, 0), (F16, 3, 130, 130, 130, 2, 0),
                                                         (F32, 0, 300, 520, 160, 0, 2)])
def test_fallback_path_matches_the_oracle(dtype, layout, M, N, K, opad, pad):
    check(M, N, K, layout, dtype, 4200 + N, 1, opad=opad, pad=pad)


def test_rows_with_a_large_mean_and_a_small_spread():
    # bias 1000 + noise: the statistics must not cancel (slice means are merged, never sum of squares minus mean^2)
    M, N, K = 260, 1024, 256
    A = synth.normal(4300, "A", M, K) * np.float32(0.01); B = synth.normal(4300, "B", K, N)
    bias = (np.float32(1000.0) + synth.normal(4300, "bias", 1, N)[0]).astype(np.float32)
    for dtype in (BF16, F32):
        As, Bs = store(A, dtype), store(B, dtype)
        got, path, _ = run(As, Bs, bias, M, N, K, 0, dtype, 1e-5)
        assert path == 0
        ref = oracle.gemm_layernorm(As, Bs, bias, M, N, K, dtype=dtype, eps=1e-5)
        # z is near 1000, its fp32 accumulation error about 1e-4 on a spread of about 1: 1e-3 of y
        assert np.max(np.abs(got - ref)) <= 2e-3 + HALF_STEP[dtype] * 5.0


def test_closed_forms_and_degenerate_cases_on_the_gpu():
    M, N, K = 260, 512, 128
    A = synth.normal(4400, "A", M, K)
    Z = np.zeros((K, N), dtype=np.float32)
    bias = synth.normal(4400, "bias", 1, N)[0]
    want = oracle.layernorm(bias[None, :], eps=1e-5)[0]
    for dtype in (BF16, F32):
        # zero weights: every row is LayerNorm of the bias
        got, path, _ = run(store(A, dtype), store(Z, dtype), bias, M, N, K, 0, dtype, 1e-5)
        assert path == 0
        assert np.max(np.abs(got - want[None, :])) <= 3e-6 * (1 + np.abs(want).max()) + HALF_STEP[dtype] * np.abs(want).max()
        assert np.all(got == got[0:1])                                            # the same bits in every row
        # K = 0: the same through the fallback
        got0, path, _ = run(store(A[:, :0], dtype), store(Z[:0], dtype), bias, M, N, 0, 0, dtype, 1e-5)
        assert path == 1
        assert np.max(np.abs(got0 - want[None, :])) <= 3e-6 * (1 + np.abs(want).max()) + HALF_STEP[dtype] * np.abs(want).max()
        # a constant row (no bias, zero weights): zero deviations, finite because of eps
        gotc, _, _ = run(store(A, dtype), store(Z, dtype), None, M, N, K, 0, dtype, 1e-5)
        assert np.all(gotc == 0.0)
    # integer operands: z is exact, so the result is LayerNorm of the exact product up to the statistics' rounding
    Ai = synth.integers(4401, "A", 256, 64); Bi = synth.integers(4401, "B", 64, 256); bi = synth.integers(4401, "bias", 1, 256)[0]
    got, path, _ = run(store(Ai, F32), store(Bi, F32), bi, 256, 256, 64, 0, F32, 0.5)
    ref = oracle.gemm_layernorm(Ai, Bi, bi, 256, 256, 64, eps=0.5)
    assert path == 0 and np.max(np.abs(got - ref)) <= 2e-6 * (1 + np.abs(ref).max())
    # nothing to do
    ob.optiml_gemm_layernorm(0, 8, 8, None, 8, None, 8, None, None, 8, 1e-5, 0, 0)
