"""CPU oracle for C = act(A.B + bias) and for its bandwidth-bound siblings (element-wise
ReLU / sigmoid, sum, dot product, mean squared error, cross-entropy, LayerNorm) and
multi-head self-attention: ctypes front end of oracle_gemm.c, oracle_streams.c and
oracle_attention.c.

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke entry point and by
the benchmark's cpu_baseline leg; the product package never imports it, and it
imports nothing from the product package.  See oracle_gemm.c for the
definition it follows (the paper's Table 4 tasks 1, 2, 10 and the naive
row-major matmul of its case-study appendix) and its arithmetic (fp64).
"""
from __future__ import annotations

import ctypes as C
import numpy as np

from .build import build as _build

F32, BF16, F16, F8E4M3, F4E2M1, F8E5M2, F6E2M3, F6E3M2 = 0, 1, 2, 3, 4, 5, 6, 7
ACT_NONE, ACT_RELU, ACT_GELU_TANH, ACT_SILU = 0, 1, 2, 3
LAYOUT_RR, LAYOUT_RC, LAYOUT_CR, LAYOUT_CC = 0, 1, 2, 3
EW_RELU, EW_SIGMOID = 0, 1
RED_SUM, RED_DOT, RED_MSE = 0, 1, 2

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build())
        i64, vp, dp = C.c_int64, C.c_void_p, C.POINTER(C.c_double)
        L.oracle_gemm_epilogue.restype = C.c_int
        L.oracle_gemm_epilogue.argtypes = [i64, i64, i64, i64, vp, i64, i64, vp, i64, i64,
                                           vp, i64, vp, vp, C.c_int, C.c_int, C.c_int]
        L.oracle_gemm_epilogue_sampled.restype = C.c_int
        L.oracle_gemm_epilogue_sampled.argtypes = [i64, vp, vp, vp, i64, i64, i64, i64,
                                                   vp, i64, i64, vp, i64, i64, vp, i64, vp, vp,
                                                   C.c_int, C.c_int, C.c_int]
        L.oracle_act.restype = C.c_double
        L.oracle_act.argtypes = [C.c_double, C.c_int]
        L.oracle_bf16_from_double.restype = C.c_uint16
        L.oracle_bf16_from_double.argtypes = [C.c_double]
        L.oracle_f16_from_double.restype = C.c_uint16
        L.oracle_f16_from_double.argtypes = [C.c_double]
        L.oracle_f16_to_double.restype = C.c_double
        L.oracle_f16_to_double.argtypes = [C.c_uint16]
        L.oracle_f8e4m3_to_double.restype = C.c_double
        L.oracle_f8e4m3_to_double.argtypes = [C.c_uint8]
        L.oracle_f8e5m2_to_double.restype = C.c_double
        L.oracle_f8e5m2_to_double.argtypes = [C.c_uint8]
        L.oracle_f4e2m1_to_double.restype = C.c_double
        L.oracle_f4e2m1_to_double.argtypes = [C.c_uint8]
        for f in (L.oracle_f6e2m3_to_double, L.oracle_f6e3m2_to_double):
            f.restype = C.c_double
            f.argtypes = [C.c_uint8]
        L.oracle_e8m0_to_double.restype = C.c_double
        L.oracle_e8m0_to_double.argtypes = [C.c_uint8]
        L.oracle_gemm_epilogue_mx.restype = C.c_int
        L.oracle_gemm_epilogue_mx.argtypes = [i64, i64, i64, vp, i64, vp, vp, i64, vp, vp, vp, C.c_int, C.c_int, C.c_int]
        L.oracle_num_threads.restype = C.c_int
        L.oracle_elementwise.restype = None
        L.oracle_elementwise.argtypes = [i64, vp, C.c_int, vp]
        L.oracle_reduce.restype = C.c_double
        L.oracle_reduce.argtypes = [i64, vp, vp, C.c_int]
        L.oracle_cross_entropy.restype = C.c_double
        L.oracle_cross_entropy.argtypes = [i64, i64, vp, vp]
        L.oracle_cross_entropy_f64.restype = C.c_double
        L.oracle_cross_entropy_f64.argtypes = [i64, i64, vp, vp]
        L.oracle_cross_entropy_rows_f64.restype = None
        L.oracle_cross_entropy_rows_f64.argtypes = [i64, i64, vp, vp, vp]
        L.oracle_layernorm_f64.restype = None
        L.oracle_layernorm_f64.argtypes = [i64, i64, vp, C.c_double, vp]
        L.oracle_transpose.restype = None
        L.oracle_transpose.argtypes = [i64, i64, vp, vp, i64]
        L.oracle_layernorm.restype = None
        L.oracle_layernorm.argtypes = [i64, i64, vp, C.c_double, vp]
        L.oracle_mhsa.restype = C.c_int
        L.oracle_mhsa.argtypes = [i64, i64, i64, i64, vp, vp, vp, C.c_int, vp]
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _check_operand(x, dtype, what):
    want = {F32: np.float32, F8E4M3: np.uint8, F4E2M1: np.uint8, F8E5M2: np.uint8, F6E2M3: np.uint8, F6E3M2: np.uint8}.get(dtype, np.uint16)
    if x.dtype != want or not x.flags.c_contiguous:
        raise TypeError(f"{what}: need C-contiguous {want.__name__} storage, got {x.dtype}")


def _geometry(A, B, layout, batch, M, N, K, lda, ldb, strideA, strideB, dtype=F32):
    """Leading dimensions / strides default to those of dense [batch, rows, ld] arrays."""
    a_col, b_col = (layout >> 1) & 1, layout & 1
    # leading dimensions in elements: E2M1 has two elements to a byte, the 6-bit types four to three bytes
    num, den = (2, 1) if dtype == F4E2M1 else (4, 3) if dtype in (F6E2M3, F6E3M2) else (1, 1)
    if lda is None:
        lda = A.shape[-1] * num // den
    if ldb is None:
        ldb = B.shape[-1] * num // den
    if strideA is None:
        strideA = (K if a_col else M) * lda if batch > 1 else 0
    if strideB is None:
        strideB = (N if b_col else K) * ldb if batch > 1 else 0
    return lda, ldb, strideA, strideB


def gemm_epilogue(A, B, bias, M, N, K, *, dtype=F32, act=ACT_NONE, layout=LAYOUT_RR, batch=1,
                  lda=None, ldb=None, strideA=None, strideB=None, strideBias=None,
                  want_absden=False):
    """Y[batch, M, N] (fp64) = act(A.B + bias); optionally also |bias| + sum|a b|."""
    _check_operand(A, dtype, "A"); _check_operand(B, dtype, "B")
    lda, ldb, strideA, strideB = _geometry(A, B, layout, batch, M, N, K, lda, ldb, strideA, strideB, dtype)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        if strideBias is None:
            strideBias = N if (batch > 1 and bias.size >= batch * N) else 0
    else:
        strideBias = 0
    Y = np.empty((batch, M, N), dtype=np.float64)
    D = np.empty((batch, M, N), dtype=np.float64) if want_absden else None
    rc = lib().oracle_gemm_epilogue(batch, M, N, K, _ptr(A), lda, strideA, _ptr(B), ldb, strideB,
                                    _ptr(bias), strideBias, _ptr(Y), _ptr(D), layout, dtype, act)
    if rc != 0:
        raise ValueError("oracle_gemm_epilogue rejected its arguments")
    return (Y, D) if want_absden else Y


def gemm_epilogue_sampled(sb, si, sj, A, B, bias, M, N, K, *, dtype=F32, act=ACT_NONE,
                          layout=LAYOUT_RR, batch=1, lda=None, ldb=None, strideA=None,
                          strideB=None, strideBias=None, want_absden=False):
    """The same definition evaluated only at entries (sb[t], si[t], sj[t])."""
    _check_operand(A, dtype, "A"); _check_operand(B, dtype, "B")
    lda, ldb, strideA, strideB = _geometry(A, B, layout, batch, M, N, K, lda, ldb, strideA, strideB, dtype)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        if strideBias is None:
            strideBias = N if (batch > 1 and bias.size >= batch * N) else 0
    else:
        strideBias = 0
    sb = np.ascontiguousarray(sb, dtype=np.int64)
    si = np.ascontiguousarray(si, dtype=np.int64)
    sj = np.ascontiguousarray(sj, dtype=np.int64)
    Y = np.empty(sb.shape[0], dtype=np.float64)
    D = np.empty(sb.shape[0], dtype=np.float64) if want_absden else None
    rc = lib().oracle_gemm_epilogue_sampled(sb.shape[0], _ptr(sb), _ptr(si), _ptr(sj), batch, M, N, K,
                                            _ptr(A), lda, strideA, _ptr(B), ldb, strideB,
                                            _ptr(bias), strideBias, _ptr(Y), _ptr(D), layout, dtype, act)
    if rc != 0:
        raise ValueError("oracle_gemm_epilogue_sampled rejected its arguments")
    return (Y, D) if want_absden else Y


def act(z, kind):
    f = lib().oracle_act
    return np.vectorize(lambda v: f(float(v), kind), otypes=[np.float64])(np.asarray(z, dtype=np.float64))


def bf16_from_double(y):
    """uint16 bit patterns of the bf16 nearest (ties to even) to each fp64 value."""
    f = lib().oracle_bf16_from_double
    return np.vectorize(lambda v: f(float(v)), otypes=[np.uint16])(np.asarray(y, dtype=np.float64))


def f16_from_double(y):
    """uint16 bit patterns of the IEEE binary16 nearest (ties to even) to each fp64 value."""
    f = lib().oracle_f16_from_double
    return np.vectorize(lambda v: f(float(v)), otypes=[np.uint16])(np.asarray(y, dtype=np.float64))


def f8e4m3_to_double(bits):
    """fp64 value of each OCP E4M3 bit pattern (uint8)."""
    f = lib().oracle_f8e4m3_to_double
    return np.vectorize(lambda b: f(int(b)), otypes=[np.float64])(np.asarray(bits, dtype=np.uint8))


def f8e5m2_to_double(bits):
    """fp64 value of each OCP E5M2 bit pattern (uint8)."""
    f = lib().oracle_f8e5m2_to_double
    return np.vectorize(lambda b: f(int(b)), otypes=[np.float64])(np.asarray(bits, dtype=np.uint8))


def f4e2m1_to_double(nibbles):
    """fp64 value of each OCP E2M1 code (low four bits of each uint8)."""
    f = lib().oracle_f4e2m1_to_double
    return np.vectorize(lambda b: f(int(b)), otypes=[np.float64])(np.asarray(nibbles, dtype=np.uint8))


def f6e2m3_to_double(codes):
    """fp64 value of each OCP E2M3 code (low six bits of each uint8)."""
    f = lib().oracle_f6e2m3_to_double
    return np.vectorize(lambda b: f(int(b)), otypes=[np.float64])(np.asarray(codes, dtype=np.uint8))


def f6e3m2_to_double(codes):
    """fp64 value of each OCP E3M2 code (low six bits of each uint8)."""
    f = lib().oracle_f6e3m2_to_double
    return np.vectorize(lambda b: f(int(b)), otypes=[np.float64])(np.asarray(codes, dtype=np.uint8))


def e8m0_to_double(codes):
    """fp64 value 2^(e - 127) of each OCP E8M0 scale code (255: NaN)."""
    f = lib().oracle_e8m0_to_double
    return np.vectorize(lambda b: f(int(b)), otypes=[np.float64])(np.asarray(codes, dtype=np.uint8))


def gemm_epilogue_mx(A, scaleA, B, scaleB, bias, M, N, K, *, dtype=F4E2M1, act=ACT_NONE, layout=LAYOUT_RC, lda=None, ldb=None):
    """Y[M, N] (fp64) = act((sA * A).(sB * B) + bias) for block-scaled operands: E4M3, E5M2, E2M3, E3M2 or E2M1 elements (uint8
    storage; E2M1 two to a byte, the 6-bit types four to three bytes) with one E8M0 scale per 32 consecutive k of every row of A (scaleA [M, ceil(K/32)]) and every column of
    B (scaleB [N, ceil(K/32)])."""
    _check_operand(A, dtype, "A"); _check_operand(B, dtype, "B")
    lda, ldb, _, _ = _geometry(A, B, layout, 1, M, N, K, lda, ldb, 0, 0, dtype)
    scaleA = np.ascontiguousarray(scaleA, dtype=np.uint8); scaleB = np.ascontiguousarray(scaleB, dtype=np.uint8)
    blocks = (K + 31) // 32
    if scaleA.shape != (M, blocks) or scaleB.shape != (N, blocks):
        raise ValueError("scales [M, ceil(K/32)] and [N, ceil(K/32)] expected")
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    Y = np.empty((M, N), dtype=np.float64)
    if lib().oracle_gemm_epilogue_mx(M, N, K, _ptr(A), lda, _ptr(scaleA), _ptr(B), ldb, _ptr(scaleB), _ptr(bias), _ptr(Y),
                                     layout, dtype, act) != 0:
        raise ValueError("oracle_gemm_epilogue_mx rejected its arguments")
    return Y


def f16_to_double(bits):
    """fp64 value of each binary16 bit pattern."""
    f = lib().oracle_f16_to_double
    return np.vectorize(lambda b: f(int(b)), otypes=[np.float64])(np.asarray(bits, dtype=np.uint16))


def elementwise(x, op):
    """fp64 array of op(x_i) for a contiguous fp32 array x (Table 4, tasks 10 and 1)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    y = np.empty(x.shape, dtype=np.float64)
    lib().oracle_elementwise(x.size, _ptr(x), op, _ptr(y))
    return y


def reduce(x, y, op):
    """fp64 value of sum(x), dot(x, y) or mean((x - y)^2) for contiguous fp32 arrays (Table 4,
    tasks 14, 15, 7); y is ignored for the sum."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if op != RED_SUM:
        y = np.ascontiguousarray(y, dtype=np.float32)
        if y.size != x.size:
            raise ValueError("operands of different length")
    return float(lib().oracle_reduce(x.size, _ptr(x), None if op == RED_SUM else _ptr(y), op))


def cross_entropy(z, labels):
    """fp64 mean over rows of log(sum_k exp(z_jk)) - z_{j, label_j} for fp32 logits [N, C] and int32
    labels [N] (Table 4, task 17)."""
    z = np.ascontiguousarray(z, dtype=np.float32)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    if z.ndim != 2 or labels.shape != (z.shape[0],):
        raise ValueError("logits [N, C] and labels [N] expected")
    return float(lib().oracle_cross_entropy(z.shape[0], z.shape[1], _ptr(z), _ptr(labels)))


def gemm_cross_entropy(A, B, bias, labels, M, N, K, *, dtype=F32, layout=LAYOUT_RR):
    """Mean over the M rows of log(sum_j exp(z_ij)) - z_{i, label_i} for the logits z = A.B + bias of the
    contraction (task 2 feeding task 17 of Table 4), every step in fp64: the logits are never rounded."""
    z = gemm_epilogue(A, B, bias, M, N, K, dtype=dtype, act=ACT_NONE, layout=layout)[0]
    z = np.ascontiguousarray(z, dtype=np.float64)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    if labels.shape != (M,):
        raise ValueError("labels [M] expected")
    return float(lib().oracle_cross_entropy_f64(M, N, _ptr(z), _ptr(labels)))


def gemm_cross_entropy_rows(A, B, bias, labels, M, N, K, *, dtype=F32, layout=LAYOUT_RR):
    """The M per-row losses log(sum_j exp(z_ij)) - z_{i, label_i} of the same fused operation (fp64 array [M]); their
    mean in row order is what gemm_cross_entropy returns up to the order of the additions."""
    z = gemm_epilogue(A, B, bias, M, N, K, dtype=dtype, act=ACT_NONE, layout=layout)[0]
    z = np.ascontiguousarray(z, dtype=np.float64)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    if labels.shape != (M,):
        raise ValueError("labels [M] expected")
    out = np.empty(M, dtype=np.float64)
    lib().oracle_cross_entropy_rows_f64(M, N, _ptr(z), _ptr(labels), _ptr(out))
    return out


def gemm_layernorm(A, B, bias, M, N, K, *, dtype=F32, layout=LAYOUT_RR, eps=1e-5):
    """LayerNorm (Table 4, task 4: mean and biased variance of a row, no scale or shift) of every row of
    z = A.B + bias (task 2), every step in fp64: the product is never rounded before it is normalised.  fp64 [M, N]."""
    z = gemm_epilogue(A, B, bias, M, N, K, dtype=dtype, act=ACT_NONE, layout=layout)[0]
    z = np.ascontiguousarray(z, dtype=np.float64).reshape(M, N)
    y = np.empty((M, N), dtype=np.float64)
    lib().oracle_layernorm_f64(M, N, _ptr(z), float(eps), _ptr(y))
    return y


def transpose(x):
    """The transposed copy of a 2-D array of 2- or 4-byte elements (Table 4, task 8), same dtype."""
    x = np.ascontiguousarray(x)
    if x.ndim != 2 or x.dtype.itemsize not in (2, 4):
        raise ValueError("a 2-D array of 2- or 4-byte elements expected")
    out = np.empty((x.shape[1], x.shape[0]), dtype=x.dtype)
    lib().oracle_transpose(x.shape[0], x.shape[1], _ptr(x), _ptr(out), x.dtype.itemsize)
    return out


def layernorm(x, eps=1e-5):
    """fp64 array of (x - mean) / sqrt(var + eps) per row of the fp32 array x [rows, len] (Table 4,
    task 4: every feature of one sample is one row)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if x.ndim != 2:
        raise ValueError("[rows, len] expected")
    y = np.empty(x.shape, dtype=np.float64)
    lib().oracle_layernorm(x.shape[0], x.shape[1], _ptr(x), float(eps), _ptr(y))
    return y


def mhsa(Q, K, V, heads, dtype=F32):
    """fp64 multi-head self-attention Concat_i softmax(Q_i K_i^T / sqrt(d_k)) V_i for Q, K, V of shape
    [batch, N, d_model] (or [N, d_model]) stored as fp32, or as bf16 / binary16 bit patterns (uint16) with dtype=BF16 / F16
    (Table 4, task 6)."""
    want = np.float32 if dtype == F32 else np.uint16
    Q, K, V = (np.ascontiguousarray(a, dtype=want) for a in (Q, K, V))
    if Q.shape != K.shape or Q.shape != V.shape or Q.ndim not in (2, 3):
        raise ValueError("Q, K, V of one shape [batch,] N, d_model expected")
    batch = Q.shape[0] if Q.ndim == 3 else 1
    N, d_model = Q.shape[-2:]
    out = np.empty(Q.shape, dtype=np.float64)
    if lib().oracle_mhsa(batch, N, d_model, heads, _ptr(Q), _ptr(K), _ptr(V), dtype, _ptr(out)) != 0:
        raise ValueError("oracle_mhsa rejected its arguments")
    return out


def num_threads():
    return lib().oracle_num_threads()
