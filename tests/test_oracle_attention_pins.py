"""Pins of the attention oracle (paper Table 4, task 6): special cases with closed forms, invariances of the
softmax, independence of heads and batches, and brute force in 50-digit decimal arithmetic."""
import math
from decimal import Decimal, getcontext

import numpy as np
import pytest

import oracle
from inputs import synth


def rand(seed, batch, N, d):
    return (synth.normal(seed, "q", N, d, batch=batch), synth.normal(seed, "k", N, d, batch=batch),
            synth.normal(seed, "v", N, d, batch=batch))


def test_zero_queries_give_the_mean_of_the_values():
    _, K, V = rand(1, 2, 37, 24)
    Q = np.zeros_like(K)
    out = oracle.mhsa(Q, K, V, heads=3)
    assert np.allclose(out, np.broadcast_to(V.astype(np.float64).mean(axis=1, keepdims=True), out.shape), rtol=1e-14, atol=1e-15)
    out = oracle.mhsa(K, np.zeros_like(K), V, heads=3)               # zero keys: the same
    assert np.allclose(out, np.broadcast_to(V.astype(np.float64).mean(axis=1, keepdims=True), out.shape), rtol=1e-14, atol=1e-15)


def test_single_key_and_identical_values():
    Q, K, V = rand(2, 1, 1, 16)
    assert np.array_equal(oracle.mhsa(Q, K, V, heads=2), V.astype(np.float64))       # N = 1: softmax over one key is 1
    Q, K, V = rand(3, 1, 50, 16)
    V[:] = V[:, :1, :]                                                               # every value row the same
    assert np.allclose(oracle.mhsa(Q, K, V, heads=4), V.astype(np.float64), rtol=1e-14)


def test_sharp_attention_selects_the_matching_value_row():
    # orthogonal one-hot keys scaled up: query i matches key pi(i) with score 400 / sqrt(dk), others 0
    N = dk = 16
    perm = np.array([(5 * i + 3) % N for i in range(N)])
    K = (20.0 * np.eye(N, dtype=np.float32))[None]
    Q = K[:, perm, :]
    V = synth.normal(4, "v", N, dk)[None]
    out = oracle.mhsa(Q, K, V, heads=1)
    w = math.exp(-400.0 / math.sqrt(dk))                                             # weight of each other key: e^-100
    assert np.allclose(out[0], V[0][perm].astype(np.float64), rtol=0, atol=16 * w * 4)
    # two-key closed form: scores (a, 0) -> weights sigma(a), 1 - sigma(a)
    Q2 = np.array([[[2.0, 0.0]]], dtype=np.float32); K2 = np.array([[[3.0, 0.0], [0.0, 0.0]]], dtype=np.float32)
    V2 = np.array([[[1.0, 10.0], [5.0, -2.0]]], dtype=np.float32)
    a = 6.0 / math.sqrt(2.0)
    s = 1.0 / (1.0 + math.exp(-a))
    got = oracle.mhsa(np.repeat(Q2, 2, axis=1), K2, V2, heads=1)[0, 0]
    assert got == pytest.approx([s * 1.0 + (1 - s) * 5.0, s * 10.0 + (1 - s) * -2.0], rel=1e-14)


def test_the_scale_is_one_over_sqrt_dk_per_head():
    Q, K, V = rand(5, 1, 9, 32)
    a = oracle.mhsa(Q, K, V, heads=2)                                                # dk = 16: scale 1/4
    b = oracle.mhsa(Q * np.float32(2.0), K, V, heads=8)                              # dk = 4: scale 1/2 ... differs
    # head 0 of the 2-head call over columns 0..15 equals a 1-head call on those columns alone
    c = oracle.mhsa(Q[..., :16], K[..., :16], V[..., :16], heads=1)
    assert np.array_equal(a[..., :16], c)
    # scaling Q by 4 at dk = 16 equals unscaled scores: compare with a hand-rolled softmax
    S = (Q[0, :, :16].astype(np.float64) @ K[0, :, :16].astype(np.float64).T) / 4.0
    P = np.exp(S - S.max(axis=1, keepdims=True)); P /= P.sum(axis=1, keepdims=True)
    assert np.allclose(c[0], P @ V[0, :, :16].astype(np.float64), rtol=1e-13, atol=1e-15)
    assert not np.allclose(a, b)


def test_invariances():
    Q, K, V = rand(6, 2, 33, 24)
    base = oracle.mhsa(Q, K, V, heads=3)
    perm = np.random.default_rng(0).permutation(33)
    assert np.allclose(oracle.mhsa(Q, K[:, perm], V[:, perm], heads=3), base, rtol=1e-13, atol=1e-15)    # keys and values together
    assert np.allclose(oracle.mhsa(Q[:, perm], K, V, heads=3), base[:, perm], rtol=0, atol=0)           # queries: rows move
    # adding a constant vector to every key shifts all scores of a query equally: softmax unchanged
    shift = np.zeros_like(K); shift[..., :] = synth.normal(7, "s", 1, 24)[0] * np.float32(0.5)
    Ks = (K.astype(np.float64) + shift).astype(np.float32)
    exact_shifted = np.array_equal(Ks.astype(np.float64), K.astype(np.float64) + shift)
    if exact_shifted:
        assert np.allclose(oracle.mhsa(Q, Ks, V, heads=3), base, rtol=1e-9, atol=1e-12)
    # output is a convex combination of value rows: within their range, column by column
    v = V.astype(np.float64)
    assert np.all(base <= v.max(axis=1, keepdims=True) + 1e-12) and np.all(base >= v.min(axis=1, keepdims=True) - 1e-12)
    # linear in V
    assert np.allclose(oracle.mhsa(Q, K, V * np.float32(-2.0), heads=3), -2.0 * base, rtol=1e-14)
    # batches are independent
    assert np.array_equal(oracle.mhsa(Q[1:], K[1:], V[1:], heads=3)[0], base[1])


def test_against_50_digit_decimal_arithmetic():
    getcontext().prec = 50
    N, d, heads = 5, 6, 2
    Q, K, V = rand(8, 1, N, d)
    dk = d // heads
    out = oracle.mhsa(Q, K, V, heads=heads)[0]
    D = lambda x: Decimal(float(x))
    for h in range(heads):
        cols = range(h * dk, (h + 1) * dk)
        for i in range(N):
            s = [sum(D(Q[0, i, c]) * D(K[0, n, c]) for c in cols) / Decimal(dk).sqrt() for n in range(N)]
            e = [x.exp() for x in s]
            tot = sum(e)
            for c in cols:
                ref = sum(e[n] * D(V[0, n, c]) for n in range(N)) / tot
                assert out[i, c] == pytest.approx(float(ref), rel=1e-13, abs=1e-15)


def test_bf16_inputs_are_widened_exactly_and_bad_arguments_rejected():
    Q, K, V = rand(9, 1, 12, 8)
    qb, kb, vb = (synth.f32_to_bf16_bits(a) for a in (Q, K, V))
    a = oracle.mhsa(qb, kb, vb, heads=2, dtype=oracle.BF16)
    b = oracle.mhsa(synth.bf16_bits_to_f32(qb), synth.bf16_bits_to_f32(kb), synth.bf16_bits_to_f32(vb), heads=2)
    assert np.array_equal(a, b)
    with pytest.raises(ValueError):
        oracle.mhsa(Q, K, V, heads=3)                       # 8 columns do not split into 3 heads
    with pytest.raises(ValueError):
        oracle.mhsa(Q, K[:, :5], V, heads=2)
    assert oracle.mhsa(Q[:, :0], K[:, :0], V[:, :0], heads=2).shape == (1, 0, 8)


def test_sixteen_bit_storage_is_decoded_exactly():
    """bf16 and binary16 inputs: the result is bit for bit that of the fp32 path on the decoded values (which numpy's
    own float16 / shift decode supplies), so the storage type only chooses the decoder."""
    Q = synth.normal(40, "q", 33, 48, batch=2); K = synth.normal(40, "k", 33, 48, batch=2); V = synth.normal(40, "v", 33, 48, batch=2)
    for dtype in (oracle.BF16, oracle.F16):
        bits = [synth.to_bits(a, dtype) for a in (Q, K, V)]
        dec = [synth.from_bits(b, dtype) for b in bits]
        assert np.array_equal(oracle.mhsa(*bits, 3, dtype=dtype), oracle.mhsa(*dec, 3))
    with pytest.raises(ValueError):
        oracle.mhsa(Q, K, V, 3, dtype=7)
