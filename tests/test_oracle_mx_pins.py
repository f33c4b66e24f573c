"""Pins of the oracle for 4-bit E2M1 operands and for block-scaled (microscaling) operands: an independent table of the
format's values, nibble addressing made visible by one-hot operands, reduction to the fp32 path on decoded values, the
E8M0 scale against ldexp, and the block-scaled contraction against exact rational arithmetic and closed forms."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
from inputs import synth

F4, F8, BF8 = oracle.F4E2M1, oracle.F8E4M3, oracle.F8E5M2
TABLE = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]       # the OCP E2M1 magnitudes by code (sign in bit 3)


def test_e2m1_decode_against_the_formats_table():
    got = oracle.f4e2m1_to_double(np.arange(16))
    assert list(got[:8]) == TABLE and list(got[8:]) == [-v for v in TABLE]
    assert math.copysign(1.0, got[8]) == -1.0                                   # code 8 is -0
    assert np.array_equal(oracle.f4e2m1_to_double(np.arange(16) | 0xF0), got)   # only the low four bits count
    # the generator's encoder and decoder: every code survives a round trip, ties go to the even code, 6 saturates
    codes = np.arange(16, dtype=np.uint8)
    assert np.array_equal(synth.f32_to_f4e2m1_codes(synth.f4e2m1_codes_to_f32(codes))[1:8], codes[1:8])
    assert np.array_equal(synth.f4e2m1_codes_to_f32(codes).astype(np.float64), got)
    x = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 0.26, 0.74, 100.0, -7.0, 5.01], dtype=np.float32)
    assert list(synth.f4e2m1_codes_to_f32(synth.f32_to_f4e2m1_codes(x))) == [0.0, 1.0, 1.0, 2.0, 2.0, 4.0, 4.0, 0.5, 0.5, 6.0, -6.0, 6.0]
    p = synth.pack_f4(np.array([[1, 2, 3, 15]], dtype=np.uint8))
    assert p.tolist() == [[0x21, 0xF3]] and synth.unpack_f4(p).tolist() == [[1, 2, 3, 15]]     # even index in the low four bits


def test_e8m0_scale_is_a_power_of_two():
    got = oracle.e8m0_to_double(np.arange(256))
    for e in (0, 1, 100, 126, 127, 128, 200, 254):
        assert got[e] == math.ldexp(1.0, e - 127)
    assert math.isnan(got[255])
    try:
        import torch
        ref = torch.arange(255, dtype=torch.uint8).view(torch.float8_e8m0fnu).to(torch.float64).numpy()
        assert np.array_equal(ref, got[:255])
    except (ImportError, AttributeError, RuntimeError, TypeError):
        pass                                                                    # this torch has no E8M0 view: ldexp above stands


@pytest.mark.parametrize("layout", [0, 1, 2, 3])
def test_e2m1_contraction_equals_the_fp32_path_on_decoded_values(layout):
    M, N, K = 6, 10, 12                                                         # every stored row has an even length
    A = synth.normal(90, "A", M, K) * np.float32(2.0); B = synth.normal(90, "B", K, N) * np.float32(2.0)
    bias = synth.normal(90, "bias", 1, N)[0]
    A4 = synth.to_bits(np.ascontiguousarray(A.T) if layout & 2 else A, synth.DTYPE_F4E2M1)
    B4 = synth.to_bits(np.ascontiguousarray(B.T) if layout & 1 else B, synth.DTYPE_F4E2M1)
    assert A4.dtype == np.uint8 and A4.shape[-1] * 2 == (M if layout & 2 else K)
    got = oracle.gemm_epilogue(A4, B4, bias, M, N, K, dtype=F4, layout=layout, act=oracle.ACT_SILU)[0]
    Ad = synth.from_bits(A4, synth.DTYPE_F4E2M1); Bd = synth.from_bits(B4, synth.DTYPE_F4E2M1)     # the generator's own decoder
    want = oracle.gemm_epilogue(Ad, Bd, bias, M, N, K, dtype=oracle.F32, layout=layout, act=oracle.ACT_SILU)[0]
    assert np.array_equal(got, want)
    assert set(np.abs(Ad).ravel()) <= set(TABLE) and len(set(np.abs(Ad).ravel())) >= 6


def test_one_hot_operands_make_the_nibble_order_visible():
    # row i of A holds a single 1.0 at k = i: C = B exactly; K odd positions sit in the high four bits
    K = N = 8
    A4 = synth.to_bits(np.eye(K, dtype=np.float32), synth.DTYPE_F4E2M1)
    Bv = (np.arange(K * N).reshape(K, N) % 13 % 8).astype(np.uint8)             # codes 0..7 -> distinct magnitudes
    Bf = synth.f4e2m1_codes_to_f32(Bv)
    got = oracle.gemm_epilogue(A4, synth.pack_f4(Bv), None, K, N, K, dtype=F4)[0]
    assert np.array_equal(got, Bf.astype(np.float64))
    # padded leading dimensions (in elements, even): the padding is never read
    Ap = np.full((K, K // 2 + 3), 0x77, dtype=np.uint8); Ap[:, :K // 2] = A4
    got = oracle.gemm_epilogue(Ap, synth.pack_f4(Bv), None, K, N, K, dtype=F4, lda=2 * Ap.shape[1])[0]
    assert np.array_equal(got, Bf.astype(np.float64))


@pytest.mark.parametrize("dtype", [F4, F8, BF8])
def test_block_scaled_contraction(dtype):
    sd = {F4: synth.DTYPE_F4E2M1, F8: synth.DTYPE_F8E4M3, BF8: synth.DTYPE_F8E5M2}[dtype]
    M, N, K = 5, 6, 80                                                          # two and a half blocks of 32
    A = synth.normal(91, "A", M, K) * np.float32(50.0); B = synth.normal(91, "B", K, N) * np.float32(0.01)
    Aq, sA = synth.mx_quantize(A, sd); Bq, sB = synth.mx_quantize(np.ascontiguousarray(B.T), sd)       # B stored [N][K]
    assert sA.shape == (M, 3) and sB.shape == (N, 3) and len(set(sA.ravel())) > 1 and sA.min() > sB.max()
    bias = synth.normal(91, "bias", 1, N)[0]
    got = oracle.gemm_epilogue_mx(Aq, sA, Bq, sB, bias, M, N, K, dtype=dtype, act=oracle.ACT_RELU)
    # exact rational arithmetic on the generator's decoded values, k descending
    Ad = synth.from_bits(Aq, sd).astype(np.float64); Bd = synth.from_bits(Bq, sd).astype(np.float64)
    for i in range(M):
        for j in range(N):
            z = sum((Fraction(float(Ad[i, k])) * Fraction(2) ** (int(sA[i, k // 32]) - 127) *
                     Fraction(float(Bd[j, k])) * Fraction(2) ** (int(sB[j, k // 32]) - 127) for k in reversed(range(K))),
                    Fraction(float(bias[j])))
            assert got[i, j] == pytest.approx(max(float(z), 0.0), rel=1e-14, abs=1e-300)
    # the quantised operands are close to what was quantised (the scales are the right powers of two)
    back = Ad * np.exp2(sA.astype(np.float64) - 127).repeat(32, axis=1)[:, :K]
    assert np.max(np.abs(back - A)) <= {F4: 0.26, F8: 0.07, BF8: 0.13}[dtype] * np.abs(A).max()
    # unit scales: the unscaled contraction of the same stored elements
    one = np.full_like(sA, 127); oneB = np.full_like(sB, 127)
    plain = oracle.gemm_epilogue(Aq, Bq, bias, M, N, K, dtype=dtype, layout=oracle.LAYOUT_RC, act=oracle.ACT_RELU)[0]
    assert np.array_equal(oracle.gemm_epilogue_mx(Aq, one, Bq, oneB, bias, M, N, K, dtype=dtype, act=oracle.ACT_RELU), plain)
    # doubling one block's scale of one row of A adds that block's partial sum once more
    up = one.copy(); up[2, 1] += 1
    z1 = oracle.gemm_epilogue_mx(Aq, one, Bq, oneB, None, M, N, K, dtype=dtype)
    z2 = oracle.gemm_epilogue_mx(Aq, up, Bq, oneB, None, M, N, K, dtype=dtype)
    part = Ad[2, 32:64] @ Bd[:, 32:64].T
    assert np.allclose(z2[2] - z1[2], part, rtol=1e-12, atol=1e-12) and np.array_equal(np.delete(z2, 2, 0), np.delete(z1, 2, 0))
    # a NaN scale poisons exactly its row (of A) or column (of B)
    bad = one.copy(); bad[4, 0] = 255
    zn = oracle.gemm_epilogue_mx(Aq, bad, Bq, oneB, None, M, N, K, dtype=dtype)
    assert np.all(np.isnan(zn[4])) and not np.any(np.isnan(zn[:4]))
    # other layouts address the same elements: A column-major, B row-major
    if dtype != F4:
        At = np.ascontiguousarray(Aq.T); Bt = np.ascontiguousarray(Bq.T)
        assert np.array_equal(oracle.gemm_epilogue_mx(At, sA, Bt, sB, bias, M, N, K, dtype=dtype, layout=oracle.LAYOUT_CR,
                                                      act=oracle.ACT_RELU), got)
