"""Pins of the oracle for 4-bit E2M1 and 6-bit E2M3 / E3M2 operands and for block-scaled (microscaling) operands: an independent table of the
format's values, nibble addressing made visible by one-hot operands, reduction to the fp32 path on decoded values, the
E8M0 scale against ldexp, and the block-scaled contraction against exact rational arithmetic and closed forms."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
from inputs import synth

F4, F8, BF8, F6, BF6 = oracle.F4E2M1, oracle.F8E4M3, oracle.F8E5M2, oracle.F6E2M3, oracle.F6E3M2
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


def _f6_value(code, ebits, mbits):
    """A 6-bit code's value from the OCP definition in exact rationals: sign, exponent field with bias 2^(ebits-1) - 1,
    fraction; exponent field 0 is subnormal; no infinities or NaNs."""
    sign = -1 if code >> 5 else 1
    e = (code >> mbits) & ((1 << ebits) - 1); f = code & ((1 << mbits) - 1)
    bias = (1 << (ebits - 1)) - 1
    if e == 0:
        return sign * Fraction(f, 1 << mbits) * Fraction(2) ** (1 - bias)
    return sign * (1 + Fraction(f, 1 << mbits)) * Fraction(2) ** (e - bias)


@pytest.mark.parametrize("dtype,ebits,mbits,largest,smallest,one", [(F6, 2, 3, 7.5, 0.125, 8), (BF6, 3, 2, 28.0, 0.0625, 12)])
def test_six_bit_decoders_against_the_format_definition(dtype, ebits, mbits, largest, smallest, one):
    dec = oracle.f6e2m3_to_double if dtype == F6 else oracle.f6e3m2_to_double
    got = dec(np.arange(64))
    assert [Fraction(float(v)) for v in got] == [_f6_value(c, ebits, mbits) for c in range(64)]
    # what the format's description fixes: largest and smallest magnitude, the code of 1.0, 32 distinct ascending magnitudes
    assert got[31] == largest and got[1] == smallest and got[one] == 1.0 and got[63] == -largest
    assert np.all(np.diff(got[:32]) > 0) and math.copysign(1.0, got[32]) == -1.0 and got[32] == 0.0
    assert np.array_equal(dec(np.arange(64) | 0xC0), got)                        # only the low six bits count
    # the generator's table (written as runs of constant spacing) is the same set of values
    sd = synth.DTYPE_F6E2M3 if dtype == F6 else synth.DTYPE_F6E3M2
    codes = np.arange(64, dtype=np.uint8)
    assert np.array_equal(synth.f6_codes_to_f32(codes, sd).astype(np.float64), got)
    back = synth.f32_to_f6_codes(synth.f6_codes_to_f32(codes, sd), sd)
    assert np.array_equal(np.delete(back, 32), np.delete(codes, 32)) and back[32] == 32      # -0 keeps its sign
    # E2M3 and E3M2 values are E4M3 values (every one of them): the 8-bit decoder, pinned elsewhere, reproduces them
    e4 = oracle.f8e4m3_to_double(np.arange(256))
    assert set(got.tolist()) <= set(e4[~np.isnan(e4)].tolist())
    # ties go to the even code, values beyond the largest saturate
    mid = (got[1:32] + got[:31]) / 2
    enc = synth.f32_to_f6_codes(mid.astype(np.float32), sd)
    assert np.all(enc % 2 == 0) and np.all(np.abs(enc.astype(int) - np.arange(31)) <= 1)
    assert synth.f32_to_f6_codes(np.array([1e9, -1e9], dtype=np.float32), sd).tolist() == [31, 63]


def test_six_bit_elements_are_a_little_endian_bit_stream():
    # codes 1, 2, 3, 63 -> bits 000001 000010 000011 111111 from bit 0 upwards = 0x81, 0x30, 0xFC
    p = synth.pack_f6(np.array([[1, 2, 3, 63]], dtype=np.uint8))
    assert p.tolist() == [[0x81, 0x30, 0xFC]] and synth.unpack_f6(p).tolist() == [[1, 2, 3, 63]]
    rng = np.random.default_rng(5)
    codes = rng.integers(0, 64, size=(7, 40), dtype=np.uint8)
    packed = synth.pack_f6(codes)
    assert packed.shape == (7, 30) and np.array_equal(synth.unpack_f6(packed), codes)
    bits = np.unpackbits(packed, axis=1, bitorder="little")                     # numpy's own bit order as the referee
    want = sum(bits[:, t::6].astype(np.uint8) << t for t in range(6))
    assert np.array_equal(want, codes)
    # one-hot A (1.0 at k = i) returns B: every position of the stream is addressed where it was packed
    for dtype, sd, one in ((F6, synth.DTYPE_F6E2M3, 8), (BF6, synth.DTYPE_F6E3M2, 12)):
        K = N = 12
        Ac = np.zeros((K, K), dtype=np.uint8); Ac[np.arange(K), np.arange(K)] = one
        Bc = ((np.arange(K * N).reshape(N, K) * 7) % 64).astype(np.uint8)       # B stored [N][K], all 64 codes occur
        got = oracle.gemm_epilogue(synth.pack_f6(Ac), synth.pack_f6(Bc), None, K, N, K, dtype=dtype, layout=oracle.LAYOUT_RC)[0]
        assert np.array_equal(got, synth.f6_codes_to_f32(Bc, sd).T.astype(np.float64))
        # padded leading dimension (in elements, a multiple of 4): the padding is never read
        Ap = np.full((K, K * 3 // 4 + 6), 0xFF, dtype=np.uint8); Ap[:, :K * 3 // 4] = synth.pack_f6(Ac)
        got = oracle.gemm_epilogue(Ap, synth.pack_f6(Bc), None, K, N, K, dtype=dtype, layout=oracle.LAYOUT_RC, lda=Ap.shape[1] * 4 // 3)[0]
        assert np.array_equal(got, synth.f6_codes_to_f32(Bc, sd).T.astype(np.float64))


@pytest.mark.parametrize("dtype", [F6, BF6])
@pytest.mark.parametrize("layout", [0, 1, 2, 3])
def test_six_bit_contraction_equals_the_fp32_path_on_decoded_values(dtype, layout):
    sd = synth.DTYPE_F6E2M3 if dtype == F6 else synth.DTYPE_F6E3M2
    M, N, K = 8, 12, 20                                                         # every stored row is a multiple of four long
    A = synth.normal(92, "A", M, K) * np.float32(2.0); B = synth.normal(92, "B", K, N) * np.float32(2.0)
    bias = synth.normal(92, "bias", 1, N)[0]
    A6 = synth.to_bits(np.ascontiguousarray(A.T) if layout & 2 else A, sd)
    B6 = synth.to_bits(np.ascontiguousarray(B.T) if layout & 1 else B, sd)
    assert A6.dtype == np.uint8 and A6.shape[-1] * 4 == 3 * (M if layout & 2 else K)
    got = oracle.gemm_epilogue(A6, B6, bias, M, N, K, dtype=dtype, layout=layout, act=oracle.ACT_SILU)[0]
    Ad = synth.from_bits(A6, sd); Bd = synth.from_bits(B6, sd)                 # the generator's own decoder
    want = oracle.gemm_epilogue(Ad, Bd, bias, M, N, K, dtype=oracle.F32, layout=layout, act=oracle.ACT_SILU)[0]
    assert np.array_equal(got, want)
    assert len(set(np.abs(Ad).ravel())) >= 12 and np.abs(Ad - (A.T if layout & 2 else A)).max() <= (0.26 if dtype == F6 else 0.51)


@pytest.mark.parametrize("dtype", [F4, F8, BF8, F6, BF6])
def test_block_scaled_contraction(dtype):
    sd = {F4: synth.DTYPE_F4E2M1, F8: synth.DTYPE_F8E4M3, BF8: synth.DTYPE_F8E5M2, F6: synth.DTYPE_F6E2M3, BF6: synth.DTYPE_F6E3M2}[dtype]
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
    assert np.max(np.abs(back - A)) <= {F4: 0.26, F8: 0.07, BF8: 0.13, F6: 0.07, BF6: 0.13}[dtype] * np.abs(A).max()
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
    # other layouts address the same elements: A column-major, B row-major (one stored element per byte only: a
    # transposed byte array of packed codes is not the transposed matrix)
    if dtype in (F8, BF8):
        At = np.ascontiguousarray(Aq.T); Bt = np.ascontiguousarray(Bq.T)
        assert np.array_equal(oracle.gemm_epilogue_mx(At, sA, Bt, sB, bias, M, N, K, dtype=dtype, layout=oracle.LAYOUT_CR,
                                                      act=oracle.ACT_RELU), got)
