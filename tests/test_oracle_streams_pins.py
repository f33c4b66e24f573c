"""Pins of the oracle for the streaming siblings (paper Table 4, tasks 1, 7, 10, 14, 15):
closed forms, invariants and independent exact arithmetic, chosen so that a dropped element, a wrong
sign, a missing 1/n or a swapped operand fails at least one of them."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
from inputs import synth

SUM, DOT, MSE = oracle.RED_SUM, oracle.RED_DOT, oracle.RED_MSE


def exact(terms):
    """Exact rational sum of fp64 terms that are themselves exact."""
    return sum((Fraction(float(t)) for t in terms), Fraction(0))


@pytest.mark.parametrize("n", [0, 1, 2, 3, 65535, 65536, 65537, 200003])
def test_sum_of_consecutive_integers_is_gauss(n):
    x = np.arange(1, n + 1, dtype=np.float32)          # exact in fp32 up to 2^24
    assert oracle.reduce(x, None, SUM) == n * (n + 1) / 2


def test_alternating_signs_catch_a_lost_or_doubled_element():
    for n in (1, 2, 65536, 65537, 131073):
        x = np.where(np.arange(n) % 2 == 0, 1.0, -1.0).astype(np.float32)
        assert oracle.reduce(x, None, SUM) == float(n % 2)


def test_dot_closed_forms_and_symmetry():
    n = 70001
    i = np.arange(n, dtype=np.float32)
    ones = np.ones(n, dtype=np.float32)
    assert oracle.reduce(i, ones, DOT) == n * (n - 1) / 2
    assert oracle.reduce(i, i, DOT) == (n - 1) * n * (2 * n - 1) / 6        # sum of squares, < 2^53
    a = synth.normal(11, "a", 1, n)[0]; b = synth.normal(11, "b", 1, n)[0]
    assert oracle.reduce(a, b, DOT) == oracle.reduce(b, a, DOT)
    assert oracle.reduce(a, -b, DOT) == -oracle.reduce(a, b, DOT)
    e = np.zeros(n, dtype=np.float32); e[12345] = 1.0
    assert oracle.reduce(a, e, DOT) == float(a[12345])                        # picks one element


def test_mse_closed_forms():
    n = 100000
    x = synth.uniform(12, "x", 1, n)[0]
    assert oracle.reduce(x, x, MSE) == 0.0
    c = np.float32(0.5)
    y = (x.astype(np.float64) + 0.5).astype(np.float32)
    d = (x.astype(np.float64) - y.astype(np.float64))                         # exact differences
    assert oracle.reduce(x, y, MSE) == pytest.approx(float(np.mean(d * d)), rel=1e-13)
    z = np.zeros(n, dtype=np.float32)
    const = np.full(n, 3.0, dtype=np.float32)
    assert oracle.reduce(const, z, MSE) == 9.0                                 # the 1/n is there
    assert oracle.reduce(z, const, MSE) == 9.0                                 # and the square
    assert oracle.reduce(np.zeros(0, np.float32), np.zeros(0, np.float32), MSE) == 0.0
    one = np.zeros(n, dtype=np.float32); one[-1] = 2.0                         # the last element counts
    assert oracle.reduce(one, z, MSE) == 4.0 / n


@pytest.mark.parametrize("n", [1, 17, 4097, 70000])
def test_reductions_against_exact_rational_arithmetic(n):
    a = synth.normal(20 + n, "a", 1, n)[0]; b = synth.normal(20 + n, "b", 1, n)[0]
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    ref = float(exact(a64))
    assert oracle.reduce(a, None, SUM) == pytest.approx(ref, abs=1e-12 * float(np.sum(np.abs(a64))))
    ref = float(exact(a64 * b64))                                              # products exact in fp64
    assert oracle.reduce(a, b, DOT) == pytest.approx(ref, abs=1e-12 * float(np.sum(np.abs(a64 * b64))))
    ref = float(sum((Fraction(float(p)) - Fraction(float(q))) ** 2 for p, q in zip(a64, b64)) / n)
    assert oracle.reduce(a, b, MSE) == pytest.approx(ref, rel=1e-12)


def test_sum_matches_math_fsum_on_a_large_array_with_cancellation():
    n = 1 << 20
    x = (synth.normal(30, "x", 1, n)[0].astype(np.float64) * 1e6).astype(np.float32)
    x[::2] = -x[1::2]                                                          # exact sum 0, large terms
    assert oracle.reduce(x, None, SUM) == 0.0
    y = synth.uniform(31, "y", 1, n)[0]
    ref = math.fsum(y.astype(np.float64).tolist())                             # exactly rounded sum
    assert oracle.reduce(y, None, SUM) == pytest.approx(ref, abs=4e-12 * float(np.sum(np.abs(y))))


def test_reduction_does_not_depend_on_the_thread_count_or_split():
    n = 300001
    x = synth.normal(32, "x", 1, n)[0]
    whole = oracle.reduce(x, None, SUM)
    assert whole == oracle.reduce(x.copy(), None, SUM)
    # blocks of 65,536 in order: the same by hand
    parts = [float(np.sum(x[i:i + 65536].astype(np.float64).cumsum()[-1:])) for i in range(0, n, 65536)]
    acc = 0.0
    for p in parts:
        acc += p
    assert whole == acc


def test_relu_is_exact_and_sigmoid_values():
    x = np.array([-3.5, -0.0, 0.0, 1e-30, 2.25, -1e30, 3e38, np.inf, -np.inf], dtype=np.float32)
    y = oracle.elementwise(x, oracle.EW_RELU)
    assert np.array_equal(y, np.maximum(x.astype(np.float64), 0.0))
    assert y.dtype == np.float64 and y.shape == x.shape
    s = oracle.elementwise(np.array([0.0, 1.0, -1.0, 2.0, -2.0, 20.0, -20.0, 100.0, -100.0, -800.0], np.float32),
                           oracle.EW_SIGMOID)
    # values computed by hand from exp(1) = 2.718281828459045, exp(2) = 7.38905609893065
    assert s[0] == 0.5
    assert s[1] == pytest.approx(1.0 / (1.0 + 1.0 / 2.718281828459045), rel=1e-15)      # 0.7310585786300049
    assert s[1] == pytest.approx(0.7310585786300049, rel=1e-15)
    assert s[3] == pytest.approx(0.8807970779778823, rel=1e-15)
    assert s[5] == pytest.approx(1.0 - 2.0611536181902037e-09, rel=1e-15)
    assert s[6] == pytest.approx(2.0611536181902037e-09, rel=1e-14)
    assert s[7] == 1.0 and 0.0 < s[8] < 1e-43 and s[9] == 0.0
    # sigma(x) + sigma(-x) = 1
    assert s[1] + s[2] == pytest.approx(1.0, abs=2e-16) and s[3] + s[4] == pytest.approx(1.0, abs=2e-16)


def test_sigmoid_against_60_digit_decimal_arithmetic():
    from decimal import Decimal, getcontext
    getcontext().prec = 60
    x = synth.uniform(40, "x", 1, 200)[0] * np.float32(30.0)
    s = oracle.elementwise(x, oracle.EW_SIGMOID)
    for xi, si in zip(x, s):
        ref = Decimal(1) / (Decimal(1) + (-Decimal(float(xi))).exp())
        assert si == pytest.approx(float(ref), rel=4e-16)
    assert np.all(np.diff(oracle.elementwise(np.sort(x), oracle.EW_SIGMOID)) >= 0)       # monotone


def test_elementwise_keeps_shape_and_empty_input():
    assert oracle.elementwise(np.zeros((0,), np.float32), oracle.EW_RELU).shape == (0,)
    x = synth.normal(41, "x", 7, 13)
    assert oracle.elementwise(x, oracle.EW_RELU).shape == (7, 13)


# ---- cross-entropy (Table 4, task 17) and LayerNorm (task 4) -----------------------------------
def test_cross_entropy_closed_forms():
    N, C = 1000, 37
    labels = (np.arange(N) * 7 % C).astype(np.int32)
    z = np.zeros((N, C), dtype=np.float32)
    assert oracle.cross_entropy(z, labels) == pytest.approx(math.log(C), rel=1e-15)          # uniform prediction
    z = np.full((N, C), 5.25, dtype=np.float32)
    assert oracle.cross_entropy(z, labels) == pytest.approx(math.log(C), rel=1e-14)          # shift invariance
    # one-hot logits of height t on the true class: loss = log(1 + (C-1) e^-t)
    for t in (1.0, 10.0, 50.0):
        z = np.zeros((N, C), dtype=np.float32); z[np.arange(N), labels] = t
        # (the stable form adds and subtracts t: absolute accuracy of a few ulp of t; the mean over
        # 1000 rows adds a relative 1e-14)
        assert oracle.cross_entropy(z, labels) == pytest.approx(math.log1p((C - 1) * math.exp(-t)), rel=1e-13, abs=1e-14)
    # ... and on a wrong class: loss = t + log(1 + (C-1) e^-t)
    z = np.zeros((N, C), dtype=np.float32); z[np.arange(N), (labels + 1) % C] = 10.0
    assert oracle.cross_entropy(z, labels) == pytest.approx(10.0 + math.log1p((C - 1) * math.exp(-10.0)), rel=1e-14)
    # huge logits do not overflow (the stable form)
    z = np.full((N, C), 3e38, dtype=np.float32)
    assert oracle.cross_entropy(z, labels) == pytest.approx(math.log(C), rel=1e-14)
    assert oracle.cross_entropy(np.zeros((0, 5), np.float32), np.zeros(0, np.int32)) == 0.0
    assert math.isnan(oracle.cross_entropy(np.zeros((3, 5), np.float32), np.array([0, 5, 1], np.int32)))


def test_cross_entropy_against_60_digit_decimal_arithmetic_and_mean_over_rows():
    from decimal import Decimal, getcontext
    getcontext().prec = 60
    N, C = 23, 11
    z = synth.normal(50, "z", N, C) * np.float32(4.0)
    labels = (np.arange(N) * 5 % C).astype(np.int32)
    tot = Decimal(0)
    for j in range(N):
        tot += sum(Decimal(float(v)).exp() for v in z[j]).ln() - Decimal(float(z[j, labels[j]]))
    assert oracle.cross_entropy(z, labels) == pytest.approx(float(tot / N), rel=1e-14)
    # the mean: doubling the batch with the same rows changes nothing; a single row is its own loss
    assert oracle.cross_entropy(np.vstack([z, z]), np.concatenate([labels, labels])) == pytest.approx(float(tot / N), rel=1e-14)
    one = oracle.cross_entropy(z[3:4], labels[3:4])
    assert one == pytest.approx(float(sum(Decimal(float(v)).exp() for v in z[3]).ln() - Decimal(float(z[3, labels[3]]))), rel=1e-14)
    # the label picks the column: moving it changes the loss by the logit difference
    l2 = labels.copy(); l2[0] = (l2[0] + 3) % C
    d = oracle.cross_entropy(z, l2) - oracle.cross_entropy(z, labels)
    assert d == pytest.approx((float(z[0, labels[0]]) - float(z[0, l2[0]])) / N, abs=1e-14)


def test_layernorm_invariants_and_closed_forms():
    rows, L = 5, 4099
    x = synth.normal(60, "x", rows, L) * np.float32(3.0) + np.float32(7.0)
    y = oracle.layernorm(x, eps=0.0)
    assert y.shape == x.shape and y.dtype == np.float64
    assert np.allclose(y.mean(axis=1), 0.0, atol=1e-13)
    assert np.allclose((y * y).mean(axis=1), 1.0, rtol=1e-13)                     # biased variance: divide by L
    # affine invariance: LayerNorm(a x + b) = sign(a) LayerNorm(x) when eps = 0 (powers of two keep x exact)
    y2 = oracle.layernorm(x * np.float32(-4.0), eps=0.0)
    assert np.allclose(y2, -y, rtol=1e-12, atol=1e-12)
    # rows are independent
    assert np.array_equal(oracle.layernorm(x[2:3], eps=0.0)[0], y[2])
    # two-point row: (-1, +1) exactly, then with eps: 1 / sqrt(1 + eps)
    t = np.array([[3.0, 5.0]], dtype=np.float32)
    assert np.array_equal(oracle.layernorm(t, eps=0.0), [[-1.0, 1.0]])
    assert oracle.layernorm(t, eps=3.0)[0, 1] == 0.5
    assert oracle.layernorm(t)[0, 1] == pytest.approx(1.0 / math.sqrt(1.0 + 1e-5), rel=1e-15)   # default eps 1e-5
    # constant row: zero deviations, finite because of eps
    assert np.array_equal(oracle.layernorm(np.full((1, 9), 2.5, np.float32)), np.zeros((1, 9)))
    # arithmetic progression 0..L-1: mean (L-1)/2, variance (L^2-1)/12
    ap = np.arange(1001, dtype=np.float32)[None, :]
    ya = oracle.layernorm(ap, eps=0.0)
    assert ya[0, 0] == pytest.approx(-500.0 / math.sqrt((1001 ** 2 - 1) / 12.0), rel=1e-14)
    assert ya[0, 500] == 0.0


def test_layernorm_against_exact_rational_statistics():
    L = 257
    x = synth.uniform(61, "x", 1, L) * np.float32(100.0)
    xs = [Fraction(float(v)) for v in x[0]]
    mean = sum(xs) / L
    var = sum((v - mean) ** 2 for v in xs) / L
    y = oracle.layernorm(x, eps=0.0)[0]
    for i in (0, 1, 100, 256):
        assert y[i] == pytest.approx(float(xs[i] - mean) / math.sqrt(float(var)), rel=1e-13)
    # large offset, small spread: the two-pass variance does not cancel
    big = (np.float32(1e6) + synth.uniform(62, "x", 1, L)).astype(np.float32)
    xb = [Fraction(float(v)) for v in big[0]]
    mb = sum(xb) / L; vb = sum((v - mb) ** 2 for v in xb) / L
    yb = oracle.layernorm(big, eps=0.0)[0]
    assert yb[7] == pytest.approx(float(xb[7] - mb) / math.sqrt(float(vb)), rel=1e-10)


# ---- the contraction feeding the cross-entropy (logits never rounded) -------------------------------------------
@pytest.mark.parametrize("dtype,layout", [(oracle.F32, 0), (oracle.BF16, 1), (oracle.F16, 2), (oracle.F32, 3)])
def test_fused_contraction_cross_entropy_against_library_routines(dtype, layout):
    """numpy's fp64 matmul of the decoded operands and scipy's logsumexp, neither of which the oracle calls."""
    from scipy.special import logsumexp
    M, N, K = 37, 53, 29
    A = synth.normal(70, "A", M, K); B = synth.normal(70, "B", K, N); bias = synth.normal(70, "bias", 1, N)[0]
    labels = ((11 * np.arange(M) + 3) % N).astype(np.int32)
    As = synth.to_bits(A.T if layout & 2 else A, dtype); Bs = synth.to_bits(B.T if layout & 1 else B, dtype)
    got = oracle.gemm_cross_entropy(As, Bs, bias, labels, M, N, K, dtype=dtype, layout=layout)
    Ad = synth.from_bits(synth.to_bits(A, dtype), dtype).astype(np.float64)
    Bd = synth.from_bits(synth.to_bits(B, dtype), dtype).astype(np.float64)
    z = Ad @ Bd + bias.astype(np.float64)
    want = float(np.mean(logsumexp(z, axis=1) - z[np.arange(M), labels]))
    assert got == pytest.approx(want, rel=1e-13)
    # a wrong label, a dropped bias or a transposed operand all move the value
    assert abs(oracle.gemm_cross_entropy(As, Bs, None, labels, M, N, K, dtype=dtype, layout=layout) - want) > 1e-5
    assert abs(oracle.gemm_cross_entropy(As, Bs, bias, (labels + 1) % N, M, N, K, dtype=dtype, layout=layout) - want) > 1e-5


def test_fused_contraction_cross_entropy_closed_forms():
    M, N, K = 9, 16, 8
    A = synth.normal(71, "A", M, K); Z = np.zeros((K, N), dtype=np.float32)
    labels = (np.arange(M) % N).astype(np.int32)
    # zero weights, no bias: uniform prediction, loss log N whatever the labels
    assert oracle.gemm_cross_entropy(A, Z, None, labels, M, N, K) == pytest.approx(math.log(N), rel=1e-15)
    # zero weights: the loss of the bias alone, the same for every row
    bias = synth.normal(71, "bias", 1, N)[0]
    b64 = bias.astype(np.float64)
    lse = math.log(float(np.sum(np.exp(b64 - b64.max())))) + float(b64.max())
    assert oracle.gemm_cross_entropy(A, Z, bias, labels, M, N, K) == pytest.approx(float(np.mean(lse - b64[labels])), rel=1e-13)
    # integer operands: the logits are exact in fp32, so the fp32-logit cross-entropy of the product agrees
    Ai = synth.integers(72, "A", M, K); Bi = synth.integers(72, "B", K, N); bi = synth.integers(72, "bias", 1, N)[0]
    z = oracle.gemm_epilogue(Ai, Bi, bi, M, N, K)[0]
    assert np.array_equal(z, z.astype(np.float32).astype(np.float64))
    assert oracle.gemm_cross_entropy(Ai, Bi, bi, labels, M, N, K) == pytest.approx(oracle.cross_entropy(z.astype(np.float32), labels), rel=1e-14)
    # identity weights scaled by t, one-hot rows: row i has logits t at i, 0 elsewhere; label = i
    t = 5.0
    E = np.eye(N, dtype=np.float32)
    want = math.log(math.exp(t) + N - 1) - t
    assert oracle.gemm_cross_entropy(E, (t * E).astype(np.float32), None, np.arange(N, dtype=np.int32), N, N, N) == pytest.approx(want, rel=1e-14)
    # out-of-range label: NaN; no rows: 0
    bad = labels.copy(); bad[3] = N
    assert math.isnan(oracle.gemm_cross_entropy(A, Z, None, bad, M, N, K))


@pytest.mark.parametrize("dtype,layout", [(oracle.F32, 0), (oracle.BF16, 1), (oracle.F16, 3)])
def test_fused_contraction_cross_entropy_row_losses(dtype, layout):
    from scipy.special import logsumexp
    M, N, K = 19, 37, 23
    A = synth.normal(73, "A", M, K); B = synth.normal(73, "B", K, N); bias = synth.normal(73, "bias", 1, N)[0]
    labels = ((5 * np.arange(M) + 36) % N).astype(np.int32)          # row 0 takes the last class
    As = synth.to_bits(A.T if layout & 2 else A, dtype); Bs = synth.to_bits(B.T if layout & 1 else B, dtype)
    rows = oracle.gemm_cross_entropy_rows(As, Bs, bias, labels, M, N, K, dtype=dtype, layout=layout)
    assert rows.shape == (M,) and rows.dtype == np.float64
    Ad = synth.from_bits(synth.to_bits(A, dtype), dtype).astype(np.float64)
    Bd = synth.from_bits(synth.to_bits(B, dtype), dtype).astype(np.float64)
    z = Ad @ Bd + bias.astype(np.float64)
    want = logsumexp(z, axis=1) - z[np.arange(M), labels]             # a library routine the oracle does not call
    assert np.allclose(rows, want, rtol=1e-13, atol=1e-14)
    # the mean of the rows is the scalar the other oracle function returns
    assert float(np.mean(rows)) == pytest.approx(oracle.gemm_cross_entropy(As, Bs, bias, labels, M, N, K, dtype=dtype, layout=layout), rel=1e-14)
    # a row's loss depends on its own label only; a wrong label in one row moves that row alone
    other = labels.copy(); other[4] = (other[4] + 1) % N
    rows2 = oracle.gemm_cross_entropy_rows(As, Bs, bias, other, M, N, K, dtype=dtype, layout=layout)
    assert abs(rows2[4] - rows[4]) > 1e-9 and np.array_equal(np.delete(rows2, 4), np.delete(rows, 4))
    # closed forms: zero weights -> log-sum-exp of the bias minus the label's bias, whatever the row
    Z = np.zeros_like(Bs)
    b64 = bias.astype(np.float64)
    rz = oracle.gemm_cross_entropy_rows(As, Z, bias, labels, M, N, K, dtype=dtype, layout=layout)
    assert np.allclose(rz, logsumexp(b64) - b64[labels], rtol=1e-14)
    bad = labels.copy(); bad[2] = -1
    rb = oracle.gemm_cross_entropy_rows(As, Bs, bias, bad, M, N, K, dtype=dtype, layout=layout)
    assert math.isnan(rb[2]) and np.array_equal(np.delete(rb, 2), np.delete(rows, 2))


# ---- the contraction followed by LayerNorm over each row of the product (task 2 into task 4) ------------------
@pytest.mark.parametrize("dtype,layout", [(oracle.F32, 0), (oracle.BF16, 1), (oracle.F16, 2), (oracle.F32, 3)])
def test_fused_contraction_layernorm_against_library_routines(dtype, layout):
    M, N, K = 11, 53, 29
    A = synth.normal(74, "A", M, K); B = synth.normal(74, "B", K, N); bias = synth.normal(74, "bias", 1, N)[0]
    As = synth.to_bits(A.T if layout & 2 else A, dtype); Bs = synth.to_bits(B.T if layout & 1 else B, dtype)
    eps = 1e-3
    got = oracle.gemm_layernorm(As, Bs, bias, M, N, K, dtype=dtype, layout=layout, eps=eps)
    assert got.shape == (M, N) and got.dtype == np.float64
    Ad = synth.from_bits(synth.to_bits(A, dtype), dtype).astype(np.float64)
    Bd = synth.from_bits(synth.to_bits(B, dtype), dtype).astype(np.float64)
    z = Ad @ Bd + bias.astype(np.float64)                             # numpy's matmul, mean and var: not the oracle's loops
    want = (z - z.mean(axis=1, keepdims=True)) / np.sqrt(z.var(axis=1, keepdims=True) + eps)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-13)
    # a dropped bias, a transposed operand or eps in the wrong place all move the values
    assert np.max(np.abs(oracle.gemm_layernorm(As, Bs, None, M, N, K, dtype=dtype, layout=layout, eps=eps) - want)) > 1e-3
    assert np.max(np.abs(oracle.gemm_layernorm(As, Bs, bias, M, N, K, dtype=dtype, layout=layout, eps=10 * eps) - want)) > 1e-4
    unbiased = (z - z.mean(axis=1, keepdims=True)) / np.sqrt(z.var(axis=1, ddof=1, keepdims=True) + eps)
    assert np.max(np.abs(got - unbiased)) > 1e-3                      # the variance divides by N, not N - 1


def test_fused_contraction_layernorm_closed_forms():
    M, N, K = 7, 24, 8
    A = synth.normal(75, "A", M, K); Z = np.zeros((K, N), dtype=np.float32)
    bias = synth.normal(75, "bias", 1, N)[0]
    # zero weights: every row is LayerNorm of the bias
    got = oracle.gemm_layernorm(A, Z, bias, M, N, K, eps=1e-5)
    one = oracle.layernorm(bias[None, :], eps=1e-5)[0]
    assert all(np.array_equal(got[i], one) for i in range(M))
    # integer operands: the product is exact in fp32, so LayerNorm of the rounded product agrees
    Ai = synth.integers(76, "A", M, K); Bi = synth.integers(76, "B", K, N); bi = synth.integers(76, "bias", 1, N)[0]
    z = oracle.gemm_epilogue(Ai, Bi, bi, M, N, K)[0]
    assert np.array_equal(z, z.astype(np.float32).astype(np.float64))
    assert np.array_equal(oracle.gemm_layernorm(Ai, Bi, bi, M, N, K, eps=0.5), oracle.layernorm(z.astype(np.float32), eps=0.5))
    # rank one, eps = 0: z_ij = u_i v_j, so a row is sign(u_i) LayerNorm(v) whatever |u_i| (powers of two: exact)
    u = np.array([[1.0], [-2.0], [0.25]], dtype=np.float32); v = synth.normal(77, "v", 1, N)
    r1 = oracle.gemm_layernorm(u, v, None, 3, N, 1, eps=0.0)
    lv = oracle.layernorm(v, eps=0.0)[0]
    assert np.allclose(r1[0], lv, rtol=1e-13) and np.allclose(r1[1], -lv, rtol=1e-13) and np.allclose(r1[2], lv, rtol=1e-13)
    # exact rational statistics of one row (brute force, k descending)
    Ab = synth.integers(78, "A", 1, 5, -7, 7); Bb = synth.uniform(78, "B", 5, 6); bb = synth.uniform(78, "bias", 1, 6)[0]
    zr = [sum((Fraction(float(Ab[0, k])) * Fraction(float(Bb[k, j])) for k in reversed(range(5))), Fraction(float(bb[j])))
          for j in range(6)]
    mean = sum(zr) / 6
    var = sum((t - mean) ** 2 for t in zr) / 6
    yb = oracle.gemm_layernorm(Ab, Bb, bb, 1, 6, 5, eps=0.0)[0]
    for j in range(6):
        assert yb[j] == pytest.approx(float(zr[j] - mean) / math.sqrt(float(var)), rel=1e-12)


def test_transpose_moves_every_element_to_its_mirror_position():
    # a matrix whose entries encode their own position: entry (i, j) = 1000 i + j
    rows, cols = 7, 13
    x = (1000 * np.arange(rows)[:, None] + np.arange(cols)[None, :]).astype(np.float32)
    t = oracle.transpose(x)
    assert t.shape == (cols, rows) and t.dtype == np.float32
    for i, j in ((0, 0), (0, 12), (6, 0), (6, 12), (3, 5)):
        assert t[j, i] == 1000 * i + j
    assert np.array_equal(t, x.T)                                  # numpy's view of the same thing
    assert np.array_equal(oracle.transpose(t), x)                  # an involution
    # 16-bit elements, bit patterns that are NaNs or denormals as floats: bytes are moved, not interpreted
    b = np.arange(5 * 9, dtype=np.uint16).reshape(5, 9) * np.uint16(1499) + np.uint16(0x7F80)
    assert np.array_equal(oracle.transpose(b), b.T)
    assert oracle.transpose(np.zeros((0, 4), np.float32)).shape == (4, 0)
    # a row and a column
    v = np.arange(11, dtype=np.int32).reshape(1, 11)
    assert np.array_equal(oracle.transpose(v), v.reshape(11, 1))
