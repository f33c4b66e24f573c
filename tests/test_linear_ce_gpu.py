"""Parity of the contraction fused with the cross-entropy (paper Table 4, task 2 into task 17) with the CPU oracle,
through the C-ABI.

Bar.  The loss of a row is 1-Lipschitz in its logits in the maximum norm, twice over (the log-sum-exp and the label's
logit), so an error of at most d on every logit moves the mean by at most 2 d.  The kernels accumulate products in
fp32: d <= 16 * 2^-24 * max_ij (|bias_j| + sum_k |a_ik b_kj|), the same componentwise bound the contraction's own
tests use.  The exponentials and their fp32 sums add about 1e-6 relative to a sum >= 1, i.e. about 1e-6 absolute on
the log; the final rounding to float adds half a float step of the loss.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2602_12305_amd import binding as ob
from inputs import synth
from gpu_harness import to_dev
from helpers import store

pytestmark = pytest.mark.gpu
F32, BF16, F16 = synth.DTYPE_F32, synth.DTYPE_BF16, synth.DTYPE_F16


def run(As, Bs, bias, labels, M, N, K, layout, dtype, rows=False):
    Ad, Bd = to_dev(As), to_dev(Bs)
    bd = None if bias is None else torch.from_numpy(np.ascontiguousarray(bias, dtype=np.float32)).cuda()
    ld = torch.from_numpy(np.ascontiguousarray(labels, dtype=np.int32)).cuda()
    out = torch.full((1,), 12345.0, dtype=torch.float32, device="cuda")
    ob.optiml_gemm_cross_entropy(M, N, K, Ad, As.shape[-1], Bd, Bs.shape[-1], bd, ld, out, layout, dtype)
    torch.cuda.synchronize()
    path = ob.optiml_gemm_cross_entropy_path(M, N, K, Ad, As.shape[-1], Bd, Bs.shape[-1], bd, layout, dtype)
    if not rows:
        return float(out.item()), path
    per_row = torch.full((M + 1,), 54321.0, dtype=torch.float32, device="cuda")
    out2 = torch.full((1,), 12345.0, dtype=torch.float32, device="cuda")
    ob.optiml_gemm_cross_entropy_rows(M, N, K, Ad, As.shape[-1], Bd, Bs.shape[-1], bd, ld, per_row, out2, layout, dtype)
    torch.cuda.synchronize()
    assert torch.equal(out, out2) or (math.isnan(out.item()) and math.isnan(out2.item()))     # the same mean, bit for bit
    per_row = per_row.cpu().numpy()
    assert per_row[M] == 54321.0                                         # nothing written past the M rows
    return float(out.item()), path, per_row[:M].astype(np.float64)


def check(M, N, K, layout, dtype, seed, want_path, *, use_bias=True, pad=0, scale=1.0, labels=None):
    A = synth.normal(seed, "A", M, K) * np.float32(scale); B = synth.normal(seed, "B", K, N)
    bias = synth.normal(seed, "bias", 1, N)[0] if use_bias else None
    if labels is None:
        labels = ((7919 * np.arange(M) + 3) % N).astype(np.int32)
    As = store(A, dtype, (layout >> 1) & 1, pad); Bs = store(B, dtype, layout & 1, pad)
    got, path, got_rows = run(As, Bs, bias, labels, M, N, K, layout, dtype, rows=True)
    assert path == want_path
    _, den = oracle.gemm_epilogue(As, Bs, bias, M, N, K, dtype=dtype, layout=layout, want_absden=True)
    ref_rows = oracle.gemm_cross_entropy_rows(As, Bs, bias, labels, M, N, K, dtype=dtype, layout=layout)
    ref = oracle.gemm_cross_entropy(As, Bs, bias, labels, M, N, K, dtype=dtype, layout=layout)
    tol = 2 * 16 * 2.0 ** -24 * float(den.max()) + 2e-6 + float(np.spacing(np.float32(abs(ref))))
    assert math.isfinite(got)
    assert abs(got - ref) <= tol, (got, ref, tol)
    # every row on its own: its logits' error bound, the exponentials, one rounding to float
    row_tol = 2 * 16 * 2.0 ** -24 * den.reshape(M, N).max(axis=1) + 2e-6 + np.spacing(np.abs(ref_rows).astype(np.float32)).astype(np.float64)
    worst = int(np.argmax(np.abs(got_rows - ref_rows) - row_tol))
    assert np.all(np.abs(got_rows - ref_rows) <= row_tol), (worst, got_rows[worst], ref_rows[worst], row_tol[worst], int(labels[worst]))
    again, _ = run(As, Bs, bias, labels, M, N, K, layout, dtype)
    assert again == got                                                  # bitwise repeatable
    return got, ref


@pytest.mark.parametrize("dtype", [BF16, F16])
@pytest.mark.parametrize("layout,M,N,K", [(0, 300, 520, 160), (1, 300, 515, 160), (0, 1024, 4096, 512), (1, 77, 64, 128),
                                          (0, 513, 264, 992), (1, 256, 1000, 1024), (0, 300, 520, 344), (1, 300, 515, 376)])
def test_matrix_pipe_path_matches_the_oracle(dtype, layout, M, N, K):
    check(M, N, K, layout, dtype, 3000 + N, 0)
    check(M, N, K, layout, dtype, 3100 + N, 0, use_bias=False, scale=0.25)


@pytest.mark.parametrize("layout,M,N,K", [(0, 300, 520, 160), (1, 300, 515, 160), (0, 1024, 2048, 512), (1, 77, 64, 64),
                                          (0, 513, 264, 1008), (1, 130, 1000, 2048), (0, 300, 520, 172), (1, 300, 515, 184)])
def test_fp32_matrix_pipe_path_matches_the_oracle(layout, M, N, K):
    check(M, N, K, layout, F32, 3500 + N, 0)
    check(M, N, K, layout, F32, 3600 + N, 0, use_bias=False, scale=0.25)


@pytest.mark.parametrize("dtype,layout,M,N,K,pad", [(F32, 0, 37, 53, 29, 0), (F32, 1, 40, 300, 48, 4), (F32, 2, 33, 257, 100, 0),
                                                    (F32, 3, 5, 1000, 7, 1), (BF16, 2, 64, 512, 128, 0), (F16, 0, 50, 77, 45, 0),
                                                    (BF16, 0, 20, 516, 160, 0), (F32, 0, 3, 1, 16, 0), (F16, 3, 130, 130, 130, 2)])
def test_fallback_path_matches_the_oracle(dtype, layout, M, N, K, pad):
    check(M, N, K, layout, dtype, 3200 + N, 1, pad=pad)


@pytest.mark.parametrize("dtype,layout,M,N,K,path", [(BF16, 0, 300, 520, 160, 0), (F16, 1, 300, 515, 160, 0), (F32, 0, 300, 516, 160, 0),
                                                     (F32, 1, 130, 1003, 256, 0), (BF16, 0, 600, 2120, 256, 0), (F32, 3, 37, 263, 29, 1)])
def test_every_row_with_its_label_in_the_ragged_last_slice_of_columns(dtype, layout, M, N, K, path):
    """Labels in the last, partly filled wave-wide slice of columns (64 for 16-bit storage, 32 for fp32) and in the
    last column of every full slice before it, rows in several 256-row tiles with a ragged last tile."""
    width = 32 if dtype == F32 else 64
    tail = list(range((N - 1) // width * width, N))                       # the columns of the ragged slice
    ends = list(range(width - 1, N, width)) + [0, N - 1]
    pool = np.array(tail * 3 + ends, dtype=np.int64)
    labels = pool[(5 * np.arange(M)) % len(pool)].astype(np.int32)
    assert (labels >= (N - 1) // width * width).sum() >= M // 3
    check(M, N, K, layout, dtype, 3700 + N, path, labels=labels)


def test_closed_forms_and_degenerate_cases_on_the_gpu():
    M, N, K = 260, 512, 128
    A = synth.normal(3300, "A", M, K)
    Z = np.zeros((K, N), dtype=np.float32)
    labels = (np.arange(M) % N).astype(np.int32)
    for dtype in (BF16, F32):
        got, path = run(store(A, dtype), store(Z, dtype), None, labels, M, N, K, 0, dtype)
        assert path == 0
        assert got == pytest.approx(math.log(N), abs=2e-6)                # zero weights: uniform prediction
        # K = 0: the loss of the bias alone
        bias = synth.normal(3300, "bias", 1, N)[0]
        got, path = run(store(A[:, :0], dtype), store(Z[:0], dtype), bias, labels, M, N, 0, 0, dtype)
        b64 = bias.astype(np.float64)
        lse = math.log(float(np.sum(np.exp(b64 - b64.max())))) + float(b64.max())
        assert path == 1 and got == pytest.approx(float(np.mean(lse - b64[labels])), abs=3e-6)
        # a label outside [0, N): NaN; no rows: 0
        bad = labels.copy(); bad[77] = N
        assert math.isnan(run(store(A, dtype), store(Z, dtype), None, bad, M, N, K, 0, dtype)[0])
        bad[77] = -1
        assert math.isnan(run(store(A, dtype), store(Z, dtype), None, bad, M, N, K, 0, dtype)[0])
        assert run(store(A[:0], dtype), store(Z, dtype), None, labels[:0], 0, N, K, 0, dtype)[0] == 0.0
    # sharp rows: identity-like weights, the label's logit t above the rest
    t, n = 6.0, 256
    E = np.eye(n, dtype=np.float32)
    got, path = run(store(E, BF16), store((t * E).astype(np.float32), BF16), None, np.arange(n, dtype=np.int32), n, n, n, 0, BF16)
    assert path == 0 and got == pytest.approx(math.log(math.exp(t) + n - 1) - t, abs=2e-6)


def test_large_logits_stay_finite():
    # logits of several hundred: the running maximum keeps every exponential in range
    M, N, K = 256, 768, 256
    got, ref = check(M, N, K, 0, BF16, 3400, 0, scale=30.0)
    assert got > 10.0
