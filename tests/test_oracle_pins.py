"""Pins for the CPU oracle: closed forms, exact rational brute force, integer
arithmetic, library reductions and identities.  None of these re-types the
oracle's formula; each would fail on a plausible slip (dropped k term, swapped
index, wrong leading dimension, transposed operand, bias before/after, wrong
activation constant)."""
import itertools
import math
from decimal import Decimal
from fractions import Fraction

import numpy as np
import pytest

import oracle
from inputs import synth
from helpers import act_decimal, as_real, exact_z, store

F32, BF16 = synth.DTYPE_F32, synth.DTYPE_BF16
ACTS = (synth.ACT_NONE, synth.ACT_RELU, synth.ACT_GELU_TANH, synth.ACT_SILU)


def run(A, B, bias, dtype=F32, act=synth.ACT_NONE, layout=0, pad=0, **kw):
    """Logical A [M,K], B [K,N] (fp32 values) -> oracle output [M,N] through the given storage."""
    M, K = A.shape[-2:]; N = B.shape[-1]
    a_col, b_col = (layout >> 1) & 1, layout & 1
    As = store(A, dtype, a_col, pad); Bs = store(B, dtype, b_col, pad)
    batch = A.shape[0] if A.ndim == 3 else 1
    Y = oracle.gemm_epilogue(As, Bs, bias, M, N, K, dtype=dtype, act=act, layout=layout, batch=batch, **kw)
    return Y if A.ndim == 3 else Y[0]


# ---- p1: identity ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("layout", [0, 1, 2, 3])
def test_identity_returns_B_exactly(dtype, layout):
    K, N = 37, 29
    B = synth.uniform(11, "B", K, N)
    if dtype == BF16:
        B = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(B))
    Y = run(np.eye(K, dtype=np.float32), B, None, dtype, layout=layout, pad=3)
    assert np.array_equal(Y, B.astype(np.float64))
    bias = synth.uniform(11, "bias", 1, N)[0]
    Yb = run(np.eye(K, dtype=np.float32), B, bias, dtype, layout=layout)
    assert np.array_equal(Yb, B.astype(np.float64) + bias.astype(np.float64))


# ---- p2: permutations -----------------------------------------------------------------------
@pytest.mark.parametrize("layout", [0, 1, 2, 3])
def test_permutation_selects_rows_and_columns(layout):
    rng = np.random.default_rng(5)
    K, N, M = 23, 17, 23
    pi = rng.permutation(K)
    P = np.zeros((M, K), dtype=np.float32); P[np.arange(M), pi] = 1.0
    B = synth.uniform(12, "B", K, N)
    assert np.array_equal(run(P, B, None, layout=layout, pad=5), B[pi].astype(np.float64))
    # B a permutation: C[:, j] = A[:, sigma(j)]
    A = synth.uniform(12, "A", 9, K)
    sig = rng.permutation(K)
    Q = np.zeros((K, K), dtype=np.float32); Q[sig, np.arange(K)] = 1.0
    assert np.array_equal(run(A, Q, None, layout=layout, pad=2), A[:, sig].astype(np.float64))


# ---- p3: rank-1 closed forms ----------------------------------------------------------------
@pytest.mark.parametrize("K", [1, 2, 15, 16, 17, 64, 1000, 1001])
def test_rank1_closed_forms(K):
    M, N = 5, 7
    u = np.arange(1, M + 1, dtype=np.float32); v = np.arange(-3, N - 3, dtype=np.float32)
    ones = np.ones(K, dtype=np.float32)
    # p = q = 1: z = K u_i v_j
    Y = run(np.outer(u, ones), np.outer(ones, v), None)
    assert np.array_equal(Y, K * np.outer(u, v).astype(np.float64))
    # p_k = k, q = 1: z = u_i v_j K(K-1)/2
    ramp = np.arange(K, dtype=np.float32)
    Y = run(np.outer(u, ramp), np.outer(ones, v), None)
    assert np.array_equal(Y, (K * (K - 1) // 2) * np.outer(u, v).astype(np.float64))
    # p_k = (-1)^k: z = u_i v_j * (K odd)
    alt = np.where(np.arange(K) % 2 == 0, 1.0, -1.0).astype(np.float32)
    Y = run(np.outer(u, alt), np.outer(ones, v), None)
    assert np.array_equal(Y, (K % 2) * np.outer(u, v).astype(np.float64))
    # geometric weights 2^-k against ones: sum = 2 - 2^(1-K), exact in fp64 for K <= 53
    if K <= 53:
        geo = (0.5 ** np.arange(K)).astype(np.float32)
        Y = run(np.outer(u, geo), np.outer(ones, v), None)
        assert np.array_equal(Y, (2.0 - 2.0 ** (1 - K)) * np.outer(u, v).astype(np.float64))


# ---- p4: integer-valued inputs are exact ----------------------------------------------------
@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("layout", [0, 1, 2, 3])
@pytest.mark.parametrize("act", [synth.ACT_NONE, synth.ACT_RELU])
def test_integer_inputs_match_int64_matmul(dtype, layout, act):
    batch, M, N, K = 3, 19, 33, 257
    A = synth.integers(21, "A", M, K, batch=batch); B = synth.integers(21, "B", K, N, batch=batch)
    bias = synth.integers(21, "bias", 1, N, -5, 5, batch=batch).reshape(batch, N)
    Z = np.einsum("bik,bkj->bij", A.astype(np.int64), B.astype(np.int64)) + bias.astype(np.int64)[:, None, :]
    want = np.maximum(Z, 0) if act == synth.ACT_RELU else Z
    Y = run(A, B, bias, dtype, act, layout, pad=1)
    assert np.array_equal(Y, want.astype(np.float64))


# ---- p5: brute force in exact rational arithmetic on tiny shapes ----------------------------
TINY = [(0, 3, 2), (3, 0, 2), (2, 3, 0), (1, 1, 1), (1, 5, 3), (4, 1, 7), (3, 4, 5), (7, 6, 9), (2, 9, 4)]


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("layout", [0, 1, 2, 3])
def test_tiny_shapes_against_exact_rationals(dtype, layout):
    for (M, N, K), act, use_bias in itertools.product(TINY, ACTS, (False, True)):
        A = synth.normal(31, "A", M, K); B = synth.normal(31, "B", K, N)
        bias = synth.normal(31, "bias", 1, N)[0] if use_bias else None
        As = store(A, dtype, (layout >> 1) & 1, pad=2); Bs = store(B, dtype, layout & 1, pad=1)
        Y = oracle.gemm_epilogue(As, Bs, bias, M, N, K, dtype=dtype, act=act, layout=layout)[0]
        assert Y.shape == (M, N)
        # exact values of what is stored (bf16 storage rounds the logical matrix first)
        Ar = as_real(store(A, dtype), dtype); Br = as_real(store(B, dtype), dtype)
        Z = exact_z(Ar, Br, bias)
        for i in range(M):
            for j in range(N):
                want = act_decimal(Z[i][j], act)
                # the oracle rounds K+1 times in fp64; bound from the exact sum of magnitudes
                mag = sum(abs(Ar[i, k] * Br[k, j]) for k in range(K)) + (abs(float(bias[j])) if use_bias else 0.0)
                tol = (K + 4) * 2.0 ** -52 * max(mag, abs(want)) + 1e-300
                assert abs(Y[i, j] - want) <= tol, (M, N, K, act, use_bias, i, j)


def test_K_zero_gives_activation_of_bias():
    bias = np.array([-2.0, -0.5, 0.0, 0.75, 3.0], dtype=np.float32)
    A = np.zeros((4, 0), dtype=np.float32); B = np.zeros((0, 5), dtype=np.float32)
    for act in ACTS:
        Y = oracle.gemm_epilogue(A, B, bias, 4, 5, 0, act=act)[0]
        for j in range(5):
            assert Y[0, j] == pytest.approx(act_decimal(float(bias[j]), act), rel=1e-15, abs=1e-300)
        assert np.array_equal(Y, np.broadcast_to(Y[0], (4, 5)))
    assert np.array_equal(oracle.gemm_epilogue(A, B, None, 4, 5, 0)[0], np.zeros((4, 5)))


# ---- p8: with no bias and no activation it is textbook GEMM (library dgemm) -----------------
@pytest.mark.parametrize("layout", [0, 1, 2, 3])
def test_reduces_to_blas_dgemm(layout):
    M, N, K = 61, 83, 129
    A = synth.uniform(41, "A", M, K); B = synth.uniform(41, "B", K, N)
    As = store(A, F32, (layout >> 1) & 1, 4); Bs = store(B, F32, layout & 1, 4)
    Y, D = oracle.gemm_epilogue(As, Bs, None, M, N, K, layout=layout, want_absden=True)
    Y, D = Y[0], D[0]
    ref = A.astype(np.float64) @ B.astype(np.float64)
    mag = np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64)
    assert np.all(np.abs(Y - ref) <= 4 * K * 2.0 ** -53 * mag)
    assert np.allclose(D, mag, rtol=1e-13)


# ---- leading dimensions, strides, batching --------------------------------------------------
def test_batched_equals_loop_of_singles_and_strides():
    batch, M, N, K = 3, 6, 10, 12
    A = synth.uniform(51, "A", M, K, batch=batch); B = synth.uniform(51, "B", K, N, batch=batch)
    bias = synth.uniform(51, "bias", 1, N, batch=batch).reshape(batch, N)
    Y = run(A, B, bias, act=synth.ACT_SILU)
    for b in range(batch):
        assert np.array_equal(Y[b], run(A[b], B[b], bias[b], act=synth.ACT_SILU))
    # shared bias (stride 0) and shared B (strideB = 0)
    Ys = oracle.gemm_epilogue(store(A, F32), store(B[0], F32), bias[0], M, N, K, batch=batch,
                              strideA=M * K, strideB=0, strideBias=0)
    for b in range(batch):
        assert np.array_equal(Ys[b], run(A[b], B[0], bias[0]))


def test_padding_is_never_read():
    M, N, K = 5, 6, 7
    A = synth.uniform(61, "A", M, K); B = synth.uniform(61, "B", K, N)
    for layout in range(4):
        assert np.array_equal(run(A, B, None, layout=layout, pad=0), run(A, B, None, layout=layout, pad=9))


def test_sampled_entries_match_full_and_integers():
    batch, M, N, K = 2, 40, 50, 300
    A = synth.integers(71, "A", M, K, batch=batch); B = synth.integers(71, "B", K, N, batch=batch)
    bias = synth.integers(71, "bias", 1, N, batch=batch).reshape(batch, N)
    sb, si, sj = synth.sample_entries(71, 500, batch, M, N, tile_m=16, tile_n=16)
    Z = np.einsum("bik,bkj->bij", A.astype(np.int64), B.astype(np.int64)) + bias.astype(np.int64)[:, None, :]
    for dtype, layout in itertools.product((F32, BF16), range(4)):
        As = store(A, dtype, (layout >> 1) & 1, 3); Bs = store(B, dtype, layout & 1, 2)
        ys = oracle.gemm_epilogue_sampled(sb, si, sj, As, Bs, bias, M, N, K, dtype=dtype, layout=layout, batch=batch)
        assert np.array_equal(ys, Z[sb, si, sj].astype(np.float64))
    Af = synth.normal(72, "A", M, K, batch=batch); Bf = synth.normal(72, "B", K, N, batch=batch)
    full, dfull = oracle.gemm_epilogue(Af, Bf, bias, M, N, K, batch=batch, act=synth.ACT_GELU_TANH, want_absden=True)
    ys, ds = oracle.gemm_epilogue_sampled(sb, si, sj, Af, Bf, bias, M, N, K, batch=batch,
                                          act=synth.ACT_GELU_TANH, want_absden=True)
    assert np.array_equal(ys, full[sb, si, sj]) and np.array_equal(ds, dfull[sb, si, sj])


# ---- p6: metamorphic relations --------------------------------------------------------------
def test_power_of_two_scaling_is_exact():
    M, N, K = 9, 11, 40
    A = synth.uniform(81, "A", M, K); B = synth.uniform(81, "B", K, N); bias = synth.uniform(81, "bias", 1, N)[0]
    base = run(A, B, bias, act=synth.ACT_RELU)
    for p in (-3, 1, 5):
        s = np.float32(2.0 ** p)
        assert np.array_equal(run(A * s, B, bias * s, act=synth.ACT_RELU), base * float(s))


def test_row_and_column_permutation_equivariance():
    rng = np.random.default_rng(3)
    M, N, K = 8, 9, 31
    A = synth.uniform(82, "A", M, K); B = synth.uniform(82, "B", K, N); bias = synth.uniform(82, "bias", 1, N)[0]
    base = run(A, B, bias, act=synth.ACT_SILU)
    pr, pc = rng.permutation(M), rng.permutation(N)
    assert np.array_equal(run(A[pr], B, bias, act=synth.ACT_SILU), base[pr])
    assert np.array_equal(run(A, B[:, pc], bias[pc], act=synth.ACT_SILU), base[:, pc])


def test_K_concatenation():
    M, N, K1, K2 = 6, 5, 17, 23
    A1 = synth.uniform(83, "A1", M, K1); A2 = synth.uniform(83, "A2", M, K2)
    B1 = synth.uniform(83, "B1", K1, N); B2 = synth.uniform(83, "B2", K2, N)
    whole = run(np.hstack([A1, A2]), np.vstack([B1, B2]), None)
    parts = run(A1, B1, None) + run(A2, B2, None)
    assert np.allclose(whole, parts, rtol=0, atol=1e-13)


# ---- p7: activations ------------------------------------------------------------------------
def test_activation_values_in_high_precision():
    xs = [-30.0, -3.0, -1.27846453164018, -1.0, -0.7524614201635628, -0.5, -1e-3, 0.0, 1e-3, 0.5, 1.0, 2.0, 3.0, 8.0, 30.0]
    for act in ACTS:
        got = oracle.act(xs, act)
        for x, g in zip(xs, got):
            want = act_decimal(x, act)
            assert g == pytest.approx(want, rel=4e-16, abs=1.2e-16 * abs(x) + 1e-300), (act, x)  # 1+tanh(u) cancels for x<0
    # printed textbook values: sigmoid(1) = 0.7310585786300049
    assert oracle.act([1.0], synth.ACT_SILU)[0] == pytest.approx(0.7310585786300049, rel=1e-15)
    assert oracle.act([1.0], synth.ACT_GELU_TANH)[0] == pytest.approx(0.8411919906082768, rel=1e-15)
    assert oracle.act([-3.0], synth.ACT_GELU_TANH)[0] == pytest.approx(-0.00363739208177302, abs=4e-16)


def test_activation_identities_and_limits():
    xs = np.linspace(-12, 12, 481)
    for act in (synth.ACT_SILU, synth.ACT_GELU_TANH):
        y = oracle.act(xs, act); ym = oracle.act(-xs, act)
        assert np.allclose(y - ym, xs, rtol=0, atol=4e-15)          # act(x) - act(-x) = x
        assert oracle.act([0.0], act)[0] == 0.0
        pos = oracle.act(np.linspace(0, 12, 200), act)
        assert np.all(np.diff(pos) > 0)                              # increasing for x >= 0
        assert oracle.act([40.0], act)[0] == pytest.approx(40.0, rel=1e-15)
        assert abs(oracle.act([-40.0], act)[0]) < 1e-15
        big = oracle.act([-450.0, 450.0, -150.0, 150.0], act)
        assert np.all(np.isfinite(big)) and big[1] == 450.0 and big[3] == 150.0
    # minima
    assert oracle.act([-1.27846453164018], synth.ACT_SILU)[0] == pytest.approx(-0.2784645427610738, rel=1e-14)
    assert oracle.act([-0.7524614201635628], synth.ACT_GELU_TANH)[0] == pytest.approx(-0.17004075057125406, rel=1e-14)
    # GELU's tanh form equals z * sigmoid(2u)
    z = np.linspace(-6, 6, 97)
    u = math.sqrt(2 / math.pi) * (z + 0.044715 * z ** 3)
    assert np.allclose(oracle.act(z, synth.ACT_GELU_TANH), z / (1 + np.exp(-2 * u)), rtol=0, atol=2e-16 * 8)
    relu = oracle.act([-2.0, -0.0, 0.0, 3.5], synth.ACT_RELU)
    assert list(relu) == [0.0, 0.0, 0.0, 3.5]


# ---- bf16 rounding used when comparing bf16 outputs -----------------------------------------
def test_bf16_rounding_is_nearest_even():
    # every finite bf16 value converts to itself; midpoints go to the even neighbour
    bits = np.arange(0, 0x7F80, dtype=np.uint16)
    vals = synth.bf16_bits_to_f32(bits).astype(np.float64)
    assert np.array_equal(oracle.bf16_from_double(vals), bits)
    assert np.array_equal(oracle.bf16_from_double(-vals[1:]), bits[1:] | 0x8000)
    mids = (vals[:-1] + vals[1:]) / 2
    want = np.where(bits[:-1] % 2 == 0, bits[:-1], bits[1:])
    assert np.array_equal(oracle.bf16_from_double(mids), want)
    eps = np.abs(vals[1:] - vals[:-1]) * 2.0 ** -20
    assert np.array_equal(oracle.bf16_from_double(mids - eps), bits[:-1])
    assert np.array_equal(oracle.bf16_from_double(mids + eps), bits[1:])
    # overflow, infinities, NaN, signed zero
    top = float(synth.bf16_bits_to_f32(np.array([0x7F7F], dtype=np.uint16))[0])
    assert oracle.bf16_from_double([top * (1 + 2.0 ** -9)])[0] == 0x7F7F
    assert oracle.bf16_from_double([top * (1 + 2.0 ** -8)])[0] == 0x7F80
    assert list(oracle.bf16_from_double([np.inf, -np.inf, -0.0])) == [0x7F80, 0xFF80, 0x8000]
    assert oracle.bf16_from_double([np.nan])[0] & 0x7FFF > 0x7F80
    # agrees with the (independent) integer-trick rounding of the input generator on fp32 values
    x = synth.normal(91, "x", 64, 1024, 0.0, 50.0)
    assert np.array_equal(oracle.bf16_from_double(x.astype(np.float64)), synth.f32_to_bf16_bits(x))


# ---- IEEE binary16 storage: decode and rounding against numpy's float16 (an independent implementation) ----
def test_f16_decode_and_rounding_agree_with_ieee_binary16():
    bits = np.arange(0, 1 << 16, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = oracle.f16_to_double(bits)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan) and np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))
    # landmarks of the format, typed by hand: largest finite, smallest normal, smallest subnormal, one, -2
    assert list(oracle.f16_to_double([0x7BFF, 0x0400, 0x0001, 0x3C00, 0xC000])) == [65504.0, 2.0 ** -14, 2.0 ** -24, 1.0, -2.0]
    # every non-NaN value rounds to itself
    assert np.array_equal(oracle.f16_from_double(got[~nan]), bits[~nan])
    # midpoints between neighbours go to the even one, a hair to either side goes to that side
    pos = bits[:0x7C00]
    v = got[:0x7C00]
    mids = (v[:-1] + v[1:]) / 2
    assert np.array_equal(oracle.f16_from_double(mids), np.where(pos[:-1] % 2 == 0, pos[:-1], pos[1:]))
    eps = (v[1:] - v[:-1]) * 2.0 ** -20
    assert np.array_equal(oracle.f16_from_double(mids - eps), pos[:-1])
    assert np.array_equal(oracle.f16_from_double(mids + eps), pos[1:])
    # overflow threshold (65520 is the midpoint to 2^16: ties to even = infinity), specials
    assert list(oracle.f16_from_double([65519.99, 65520.0, 1e9, -1e9, np.inf, -0.0, 2.0 ** -25, 2.0 ** -25 * 1.0001])) == \
        [0x7BFF, 0x7C00, 0x7C00, 0xFC00, 0x7C00, 0x8000, 0x0000, 0x0001]
    assert oracle.f16_from_double([np.nan])[0] & 0x7FFF > 0x7C00
    # random doubles over the whole range, against numpy's double -> half conversion
    rng = np.random.default_rng(5)
    x = rng.standard_normal(20000) * np.exp2(rng.integers(-30, 17, 20000))
    with np.errstate(over="ignore"):
        assert np.array_equal(oracle.f16_from_double(x), x.astype(np.float16).view(np.uint16))


def test_f8e4m3_decode_and_the_generator_encoding_agree_with_the_ocp_format():
    import torch
    bits = np.arange(256, dtype=np.uint8)
    want = torch.from_numpy(bits.copy()).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)   # an independent decoder
    got = oracle.f8e4m3_to_double(bits)
    nan = np.isnan(want)
    assert list(np.flatnonzero(nan)) == [0x7F, 0xFF]
    assert np.array_equal(np.isnan(got), nan) and np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))
    # landmarks typed by hand: largest finite 448, smallest normal 2^-6, smallest subnormal 2^-9, one, -1.5
    assert list(oracle.f8e4m3_to_double([0x7E, 0x08, 0x01, 0x38, 0xBC])) == [448.0, 2.0 ** -6, 2.0 ** -9, 1.0, -1.5]
    # the input generator's own decoder and encoder (numpy, no code shared with the oracle)
    assert np.array_equal(synth.f8e4m3_bits_to_f32(bits)[~nan].astype(np.float64), want[~nan])
    assert np.array_equal(synth.f32_to_f8e4m3_bits(got[~nan].astype(np.float32)), bits[~nan])          # every value to itself
    x = synth.normal(93, "x", 64, 1024, 0.0, 3.0)
    enc = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(synth.f32_to_f8e4m3_bits(x), enc)                                           # in range: torch's rounding
    mids = (got[:0x7E] + got[1:0x7F]) / 2                                                             # ties go to the even neighbour
    assert np.array_equal(synth.f32_to_f8e4m3_bits(mids.astype(np.float32)), np.where(bits[:0x7E] % 2 == 0, bits[:0x7E], bits[1:0x7F]))
    assert list(synth.f32_to_f8e4m3_bits(np.array([1e9, -1e9, 464.0, np.nan, -0.0], np.float32))) == [0x7E, 0xFE, 0x7E, 0x7F, 0x80]


def test_f8e4m3_storage_reduces_to_the_fp64_product_of_the_decoded_operands():
    M, N, K = 7, 9, 33
    A = synth.to_bits(synth.normal(94, "A", M, K), oracle.F8E4M3); B = synth.to_bits(synth.normal(94, "B", N, K), oracle.F8E4M3)
    bias = synth.normal(94, "bias", 1, N)[0]
    y = oracle.gemm_epilogue(A, B, bias, M, N, K, dtype=oracle.F8E4M3, layout=synth.LAYOUT_RC)[0]
    ref = synth.f8e4m3_bits_to_f32(A).astype(np.float64) @ synth.f8e4m3_bits_to_f32(B).astype(np.float64).T + bias.astype(np.float64)
    assert np.allclose(y, ref, rtol=0, atol=1e-13)


def test_f8e5m2_decode_and_the_generator_encoding_agree_with_the_ocp_format():
    import torch
    bits = np.arange(256, dtype=np.uint8)
    want = torch.from_numpy(bits.copy()).view(torch.float8_e5m2).float().numpy().astype(np.float64)      # an independent decoder
    got = oracle.f8e5m2_to_double(bits)
    nan = np.isnan(want)
    assert list(np.flatnonzero(nan)) == [0x7D, 0x7E, 0x7F, 0xFD, 0xFE, 0xFF]
    assert np.array_equal(np.isnan(got), nan) and np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))
    # E5M2 is binary16 cut after two fraction bits: a second independent decoder
    assert np.array_equal(got[~nan], (bits.astype(np.uint16) << 8).view(np.float16).astype(np.float64)[~nan])
    # landmarks typed by hand: largest finite 57344, infinity, smallest normal 2^-14, smallest subnormal 2^-16, one, -1.5, -1.75
    assert list(oracle.f8e5m2_to_double([0x7B, 0x7C, 0x04, 0x01, 0x3C, 0xBE, 0xBF])) == [57344.0, np.inf, 2.0 ** -14, 2.0 ** -16, 1.0, -1.5, -1.75]
    # the input generator's own decoder and encoder (numpy, no code shared with the oracle)
    assert np.array_equal(synth.f8e5m2_bits_to_f32(bits)[~nan].astype(np.float64), want[~nan])
    assert np.array_equal(synth.f32_to_f8e5m2_bits(got[~nan].astype(np.float32)), bits[~nan])          # every value to itself
    x = np.concatenate([synth.normal(95, "x", 64, 1024, 0.0, 3.0).ravel(), synth.normal(96, "y", 8, 1024, 0.0, 3e-5).ravel(),
                        synth.normal(97, "z", 8, 1024, 0.0, 2e4).ravel()])
    enc = torch.from_numpy(x).to(torch.float8_e5m2).view(torch.uint8).numpy()
    assert np.array_equal(synth.f32_to_f8e5m2_bits(x), enc)                                           # torch's rounding, subnormals and overflow included
    fin = got[:0x7C]
    mids = (fin[:-1] + fin[1:]) / 2                                                                   # ties go to the even neighbour
    assert np.array_equal(synth.f32_to_f8e5m2_bits(mids.astype(np.float32)), np.where(bits[:0x7B] % 2 == 0, bits[:0x7B], bits[1:0x7C]))
    assert list(synth.f32_to_f8e5m2_bits(np.array([1e9, -1e9, 61439.0, 61440.0, np.nan, -0.0, np.inf], np.float32))) == \
        [0x7C, 0xFC, 0x7B, 0x7C, 0x7F, 0x80, 0x7C]


def test_f8e5m2_storage_reduces_to_the_fp64_product_of_the_decoded_operands():
    M, N, K = 7, 9, 33
    A = synth.to_bits(synth.normal(98, "A", M, K), oracle.F8E5M2); B = synth.to_bits(synth.normal(98, "B", N, K), oracle.F8E5M2)
    bias = synth.normal(98, "bias", 1, N)[0]
    y = oracle.gemm_epilogue(A, B, bias, M, N, K, dtype=oracle.F8E5M2, layout=synth.LAYOUT_RC)[0]
    ref = synth.f8e5m2_bits_to_f32(A).astype(np.float64) @ synth.f8e5m2_bits_to_f32(B).astype(np.float64).T + bias.astype(np.float64)
    assert np.allclose(y, ref, rtol=0, atol=1e-13)
    # the two 8-bit types are told apart: the same bytes read as E4M3 give another product
    y4 = oracle.gemm_epilogue(A, B, bias, M, N, K, dtype=oracle.F8E4M3, layout=synth.LAYOUT_RC)[0]
    assert not np.allclose(y, y4, rtol=1e-3, atol=1e-3)
    # row-major B and column-major A address the same elements
    y2 = oracle.gemm_epilogue(np.ascontiguousarray(A.T), np.ascontiguousarray(B.T), bias, M, N, K, dtype=oracle.F8E5M2, layout=2)[0]
    assert np.array_equal(y, y2)


def test_f16_storage_reduces_to_the_fp64_product_of_the_decoded_operands():
    rng = np.random.default_rng(6)
    M, N, K = 7, 9, 33
    A = rng.standard_normal((M, K)).astype(np.float16)
    B = rng.standard_normal((K, N)).astype(np.float16)
    bias = rng.standard_normal(N).astype(np.float32)
    y = oracle.gemm_epilogue(A.view(np.uint16), B.view(np.uint16), bias, M, N, K, dtype=oracle.F16)[0]
    ref = A.astype(np.float64) @ B.astype(np.float64) + bias.astype(np.float64)
    assert np.allclose(y, ref, rtol=0, atol=1e-13)
    # column-major B, batch of two, ReLU
    Bt = np.ascontiguousarray(np.stack([B.T, 2 * B.T]))
    A2 = np.ascontiguousarray(np.stack([A, A]))
    y = oracle.gemm_epilogue(A2.view(np.uint16), Bt.view(np.uint16), None, M, N, K, dtype=oracle.F16, layout=synth.LAYOUT_RC,
                             act=synth.ACT_RELU, batch=2)
    ref = np.maximum(np.stack([A.astype(np.float64) @ B.astype(np.float64), 2 * (A.astype(np.float64) @ B.astype(np.float64))]), 0)
    assert np.allclose(y, ref, rtol=0, atol=1e-13)


def test_rejects_bad_arguments():
    A = np.zeros((2, 2), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.gemm_epilogue(A, A, None, 2, 2, 2, act=9)
    with pytest.raises(ValueError):
        oracle.gemm_epilogue(A, A, None, 2, 2, 2, layout=4)
    with pytest.raises(TypeError):
        oracle.gemm_epilogue(A.astype(np.float64), A, None, 2, 2, 2)
    with pytest.raises(ValueError):
        oracle.gemm_epilogue_sampled([0], [2], [0], A, A, None, 2, 2, 2)
