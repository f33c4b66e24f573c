"""Parity of the row-wise siblings (cross-entropy and LayerNorm; paper Table 4 tasks 17 and 4) with the
CPU oracle, through the C-ABI.

Bars.  Cross-entropy: exponentials and the per-row sum are fp32 (each exponential about 2 ulp, the sum of C
positive terms a few more), so a row's log-sum-exp carries at most about 5e-7 of absolute error; z_y - max is
exact; rows are averaged in fp64: |L - ref| <= 1e-6 + one float step of ref.  LayerNorm: statistics and the
normalisation are fp64, one rounding to float: |y - ref| <= one float step of ref + 1e-6 * |ref| slack for the
shifted-data variance of the long-row path (relative error of the variance about 1e-16 * (mean - x0)^2 / var).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_12305_amd import binding as ob
from inputs import synth

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_ce(z, labels, pad=0, offset=0):
    N, C = z.shape
    ld = C + pad
    buf = torch.full((N * ld + offset + 8,), 1e30, dtype=torch.float32, device="cuda")   # padding would dominate if read
    zd = buf[offset:offset + N * ld].view(N, ld)
    zd[:, :C] = dev(z)
    ld_ = dev(labels.astype(np.int32))
    out = torch.full((3,), 7.0, dtype=torch.float32, device="cuda")
    ob.optiml_cross_entropy(N, C, buf[offset:], ld, ld_, out[1:])
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert o[0] == 7.0 and o[2] == 7.0
    return np.float32(o[1])


def check_ce(z, labels, **kw):
    got = run_ce(z, labels, **kw)
    ref = oracle.cross_entropy(z, labels)
    assert abs(float(got) - ref) <= 1e-6 + float(np.spacing(np.float32(abs(ref)))), (float(got), ref)
    assert run_ce(z, labels, **kw) == got                                           # bitwise repeatable
    return got


@pytest.mark.parametrize("N,C", [(1, 1), (5, 2), (1000, 10), (257, 63), (300, 64), (77, 100), (33, 1000), (9, 2048),
                                 (7, 2052), (5, 5000), (3, 50257), (4100, 128), (531, 68), (400, 130), (263, 256), (129, 260),
                                 (77, 512), (65, 514), (50, 1024), (41, 1022), (35, 1028)])
def test_cross_entropy_matches_the_oracle(N, C):
    z = synth.normal(1100 + N + C, "z", N, C) * np.float32(3.0)
    labels = (np.arange(N, dtype=np.int64) * 7919 % C).astype(np.int32)
    check_ce(z, labels)
    check_ce(z, labels, pad=4)                     # ld > C, rows still 16-byte aligned when C % 4 == 0
    check_ce(z, labels, pad=1, offset=1)           # unaligned rows: scalar path


def test_cross_entropy_closed_forms_on_the_gpu():
    N, C = 512, 1000
    labels = (np.arange(N) * 13 % C).astype(np.int32)
    z = np.zeros((N, C), dtype=np.float32)
    assert float(run_ce(z, labels)) == pytest.approx(np.log(C), abs=1e-6)
    z[np.arange(N), labels] = 10.0                                                   # confident and right
    assert float(run_ce(z, labels)) == pytest.approx(np.log1p((C - 1) * np.exp(-10.0)), abs=1e-6)
    z[np.arange(N), labels] = 30.0                                                   # the fp32 row sum absorbs 1e-10
    assert 0.0 <= float(run_ce(z, labels)) <= 1e-6
    z = np.full((N, C), -3e38, dtype=np.float32); z[:, 0] = 3e38                     # extreme spread, no overflow
    lab0 = np.zeros(N, dtype=np.int32)
    assert float(run_ce(z, lab0)) == 0.0
    z = synth.normal(1200, "z", N, C)
    bad = labels.copy(); bad[100] = C                                                # label outside [0, C)
    assert np.isnan(run_ce(z, bad))
    out = torch.full((1,), 7.0, dtype=torch.float32, device="cuda")
    ob.optiml_cross_entropy(0, 10, None, 10, None, out)
    torch.cuda.synchronize()
    assert out.item() == 0.0


def run_ln(x, eps, offset=0, inplace=False):
    rows, L = x.shape
    n = rows * L
    xd = torch.zeros(n + offset + 8, dtype=torch.float32, device="cuda"); xd[offset:offset + n] = dev(x.reshape(-1))
    yd = xd if inplace else torch.full((n + offset + 8,), 7.0, dtype=torch.float32, device="cuda")
    ob.optiml_layernorm(rows, L, xd[offset:], yd[offset:], eps)
    torch.cuda.synchronize()
    out = yd.cpu().numpy()
    if not inplace:
        assert np.all(out[:offset] == 7.0) and np.all(out[offset + n:] == 7.0)
    return out[offset:offset + n].reshape(rows, L)


def check_ln(x, eps=1e-5, **kw):
    got = run_ln(x, eps, **kw).astype(np.float64)
    ref = oracle.layernorm(x, eps)
    tol = np.spacing(np.abs(ref).astype(np.float32)).astype(np.float64) + 1e-6 * np.abs(ref)
    bad = np.argwhere(np.abs(got - ref) > tol)
    assert bad.size == 0, (bad[0], got[tuple(bad[0])], ref[tuple(bad[0])])


@pytest.mark.parametrize("rows,L", [(1, 1), (3, 2), (5, 7), (4, 256), (3, 1000), (11, 252), (13, 256), (6, 260), (10, 512), (9, 1024), (7, 2048), (5, 2052), (2, 8192), (2, 8196), (3, 32768), (3, 40000), (2, 65536), (2, 65540),
                                    (2, 32772), (3, 100003), (2, 1 << 20), (1, (1 << 22) + 4)])
def test_layernorm_matches_the_oracle(rows, L):
    x = synth.normal(1300 + rows + L, "x", rows, L) * np.float32(2.5) + np.float32(1.25)
    check_ln(x)
    if L < (1 << 22):
        check_ln(x, offset=1)                      # unaligned: scalar path
    check_ln(x, eps=0.0 if L > 1 else 1e-5)


def test_layernorm_offset_data_constant_rows_and_in_place():
    L = 50000
    big = (np.float32(1e6) + synth.uniform(1400, "x", 2, L)).astype(np.float32)      # |mean| >> std: no cancellation
    check_ln(big, eps=0.0)
    small = (np.float32(1e6) + synth.uniform(1401, "x", 4, 4096)).astype(np.float32)
    check_ln(small, eps=0.0)
    const = np.full((3, 20000), 2.5, dtype=np.float32)
    assert np.all(run_ln(const, 1e-5) == 0.0)
    x = synth.normal(1402, "x", 6, 3000)
    ref = oracle.layernorm(x, 1e-5)
    got = run_ln(x, 1e-5, inplace=True).astype(np.float64)
    assert np.all(np.abs(got - ref) <= np.spacing(np.abs(ref).astype(np.float32)) + 1e-6 * np.abs(ref))
    # many rows: more rows than one 64 MiB group of the long-row path holds
    many = synth.normal(1403, "x", 300, 70000)
    check_ln(many)


def test_layernorm_long_rows_do_not_depend_on_the_wait_between_workgroups():
    """Aligned long rows are normalised in one pass by workgroups that wait for each other's partial sums; a wait that
    runs out hands the chunk to the second kernel.  With the limit at 0 every workgroup that is not the last of its
    row gives up, so the second kernel does nearly all the work: same bits, same parity."""
    cases = [synth.normal(1500, "x", 3, 40000) * np.float32(2.5) + np.float32(1.25), synth.normal(1501, "x", 2, (1 << 20) + 8),
             synth.normal(1502, "x", 70, 70000)]
    try:
        for x in cases:
            ob.optiml_set_wait_limit(1 << 22)
            waited = run_ln(x, 1e-5)
            ob.optiml_set_wait_limit(0)
            gave_up = run_ln(x, 1e-5)
            assert np.array_equal(waited, gave_up)
            check_ln(x)                                 # against the oracle, still with no waiting
            ob.optiml_set_wait_limit(-5)                # counts as 0
            assert np.array_equal(run_ln(x, 1e-5, inplace=True), waited)
        # rows that take two kernels per group (not a multiple of 4 long): in place, x[row][0] is overwritten while
        # other workgroups still need it as the pivot of the row's sums
        odd = synth.normal(1503, "x", 3, 100003) + np.float32(3.0)
        assert np.array_equal(run_ln(odd, 1e-5, inplace=True), run_ln(odd, 1e-5))
    finally:
        ob.optiml_set_wait_limit(1 << 22)
