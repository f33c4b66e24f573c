"""ctypes binding of liboptiml.so: the same entry points as include/optiml.h.

Argument marshalling only.  Operands may be torch tensors on the GPU (their
data_ptr() is passed) or plain integers holding device addresses; shapes,
leading dimensions and strides are always explicit, in elements.  Nothing is
computed here and there is no fallback: if the shared library is missing, the
first call raises.
"""
from __future__ import annotations

import ctypes as C
import os

F32, BF16, F16, F8E4M3, F4E2M1, F8E5M2, F6E2M3, F6E3M2 = 0, 1, 2, 3, 4, 5, 6, 7
ACT_NONE, ACT_RELU, ACT_GELU_TANH, ACT_SILU = 0, 1, 2, 3
LAYOUT_RR, LAYOUT_RC, LAYOUT_CR, LAYOUT_CC = 0, 1, 2, 3
LAYOUT_C_COLUMN_MAJOR = 4        # added to any of the four
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_HIP = 0, -1, -2, -3

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc", "liboptiml.so")

_i64, _vp, _int = C.c_int64, C.c_void_p, C.c_int
_PROBLEM = [_i64, _i64, _i64, _i64, _vp, _i64, _i64, _vp, _i64, _i64, _vp, _i64, _vp, _i64, _i64, _int, _int, _int]

SIGNATURES = {
    "optiml_gemm_epilogue": (_int, [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _vp, _i64, _int, _int, _vp]),
    "optiml_gemm_epilogue_ex": (_int, [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _vp, _i64, _int, _int, _int, _vp]),
    "optiml_gemm_epilogue_strided_batched": (_int, _PROBLEM + [_vp]),
    "optiml_gemm_epilogue_noalloc": (_int, _PROBLEM + [_vp]),
    "optiml_variant_count": (_int, []),
    "optiml_variant_name": (C.c_char_p, [_int]),
    "optiml_select_variant": (_int, _PROBLEM),
    "optiml_variant_supports": (_int, [_int] + _PROBLEM),
    "optiml_gemm_epilogue_variant": (_int, _PROBLEM + [_vp, _int]),
    "optiml_variant_resources": (_int, [_int, C.POINTER(_int), C.POINTER(_int), C.POINTER(_int)]),
    "optiml_copy_bytes": (_int, [_vp, _vp, _i64, _vp]),
    "optiml_mfma_probe": (_int, [_vp, _i64, _vp, _i64, _i64, _int, _int, C.POINTER(C.c_double), _vp]),
    "optiml_elementwise": (_int, [_i64, _vp, _vp, _int, _vp]),
    "optiml_reduce": (_int, [_i64, _vp, _vp, _int, _vp, _vp]),
    "optiml_cross_entropy": (_int, [_i64, _i64, _vp, _i64, _vp, _vp, _vp]),
    "optiml_layernorm": (_int, [_i64, _i64, _vp, _vp, C.c_float, _vp]),
    "optiml_mhsa": (_int, [_i64, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _int, _vp]),
    "optiml_transpose": (_int, [_i64, _i64, _vp, _i64, _vp, _i64, _int, _vp]),
    "optiml_gemm_cross_entropy": (_int, [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _vp, _vp, _int, _int, _vp]),
    "optiml_gemm_cross_entropy_rows": (_int, [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _vp, _vp, _vp, _int, _int, _vp]),
    "optiml_gemm_layernorm": (_int, [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _vp, _i64, C.c_float, _int, _int, _vp]),
    "optiml_gemm_layernorm_path": (_int, [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _vp, _i64, _int, _int]),
    "optiml_gemm_cross_entropy_path": (_int, [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _int, _int]),
    "optiml_set_workspace": (_int, [_vp, _i64]),
    "optiml_workspace_bytes": (_i64, []),
    "optiml_set_wait_limit": (None, [_i64]),
    "optiml_gemm_epilogue_mx": (_int, [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _vp, _i64, _int, _int, _vp]),
    "optiml_gemm_epilogue_mx_path": (_int, [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _vp, _i64, _int]),
    "optiml_status_string": (C.c_char_p, [_int]),
    "optiml_last_hip_error": (_int, []),
}

_lib = None


class OptimlError(RuntimeError):
    def __init__(self, status):
        self.status = status
        text = lib().optiml_status_string(status).decode()
        if status == ERR_HIP:
            text += f" (hipError_t {lib().optiml_last_hip_error()})"
        super().__init__(f"optiml status {status}: {text}")


def lib():
    """The loaded shared library (opened on first use)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2602_12305_amd.csrc.build` "
                              "(there is no fallback path)")
        # PyTorch carries its own HIP runtime; load it first so that the library binds to that
        # copy (two runtimes in one process do not share a device context)
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _addr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status):
    if status != OK:
        raise OptimlError(status)
    return status


def optiml_gemm_epilogue(M, N, K, A, lda, B, ldb, bias, Cout, ldc, dtype, act, stream=None):
    return _check(lib().optiml_gemm_epilogue(M, N, K, _addr(A), lda, _addr(B), ldb, _addr(bias), _addr(Cout), ldc,
                                             dtype, act, _stream(stream)))


def optiml_gemm_epilogue_ex(M, N, K, A, lda, B, ldb, bias, Cout, ldc, layout, dtype, act, stream=None):
    return _check(lib().optiml_gemm_epilogue_ex(M, N, K, _addr(A), lda, _addr(B), ldb, _addr(bias), _addr(Cout), ldc,
                                                layout, dtype, act, _stream(stream)))


def optiml_gemm_epilogue_strided_batched(batch, M, N, K, A, lda, strideA, B, ldb, strideB, bias, strideBias,
                                         Cout, ldc, strideC, layout, dtype, act, stream=None):
    return _check(lib().optiml_gemm_epilogue_strided_batched(
        batch, M, N, K, _addr(A), lda, strideA, _addr(B), ldb, strideB, _addr(bias), strideBias,
        _addr(Cout), ldc, strideC, layout, dtype, act, _stream(stream)))


def optiml_gemm_epilogue_noalloc(batch, M, N, K, A, lda, strideA, B, ldb, strideB, bias, strideBias,
                                 Cout, ldc, strideC, layout, dtype, act, stream=None):
    return _check(lib().optiml_gemm_epilogue_noalloc(
        batch, M, N, K, _addr(A), lda, strideA, _addr(B), ldb, strideB, _addr(bias), strideBias,
        _addr(Cout), ldc, strideC, layout, dtype, act, _stream(stream)))


def optiml_gemm_epilogue_variant(batch, M, N, K, A, lda, strideA, B, ldb, strideB, bias, strideBias,
                                 Cout, ldc, strideC, layout, dtype, act, variant_id, stream=None):
    return _check(lib().optiml_gemm_epilogue_variant(
        batch, M, N, K, _addr(A), lda, strideA, _addr(B), ldb, strideB, _addr(bias), strideBias,
        _addr(Cout), ldc, strideC, layout, dtype, act, _stream(stream), variant_id))


def optiml_select_variant(batch, M, N, K, A, lda, strideA, B, ldb, strideB, bias, strideBias,
                          Cout, ldc, strideC, layout, dtype, act):
    """Variant id the dispatcher would use (>= 0) or a negative status; host logic only."""
    return lib().optiml_select_variant(batch, M, N, K, _addr(A), lda, strideA, _addr(B), ldb, strideB,
                                       _addr(bias), strideBias, _addr(Cout), ldc, strideC, layout, dtype, act)


def optiml_variant_supports(variant_id, batch, M, N, K, A, lda, strideA, B, ldb, strideB, bias, strideBias,
                            Cout, ldc, strideC, layout, dtype, act):
    return lib().optiml_variant_supports(variant_id, batch, M, N, K, _addr(A), lda, strideA, _addr(B), ldb, strideB,
                                         _addr(bias), strideBias, _addr(Cout), ldc, strideC, layout, dtype, act)


def optiml_variant_count():
    return lib().optiml_variant_count()


def optiml_variant_name(variant_id):
    s = lib().optiml_variant_name(variant_id)
    return None if s is None else s.decode()


def optiml_variant_resources(variant_id):
    """(registers per lane, scratch bytes per lane, static LDS bytes) of a variant's main kernel."""
    r, sc, l = _int(0), _int(0), _int(0)
    _check(lib().optiml_variant_resources(variant_id, C.byref(r), C.byref(sc), C.byref(l)))
    return r.value, sc.value, l.value


def optiml_copy_bytes(dst, src, nbytes, stream=None):
    return _check(lib().optiml_copy_bytes(_addr(dst), _addr(src), nbytes, _stream(stream)))


def optiml_mfma_probe(operands, operand_bytes, sink, sink_floats, iters, dtype, lds_reads=0, stream=None):
    """Enqueue the matrix-pipe rate probe; returns the number of flops the launch performs."""
    flops = C.c_double(0.0)
    _check(lib().optiml_mfma_probe(_addr(operands), operand_bytes, _addr(sink), sink_floats, iters, dtype, lds_reads,
                                   C.byref(flops), _stream(stream)))
    return flops.value


def optiml_elementwise(n, x, y, op, stream=None):
    return _check(lib().optiml_elementwise(n, _addr(x), _addr(y), op, _stream(stream)))


def optiml_reduce(n, x, y, op, out, stream=None):
    return _check(lib().optiml_reduce(n, _addr(x), _addr(y), op, _addr(out), _stream(stream)))


def optiml_cross_entropy(N, Cn, logits, ld, labels, loss, stream=None):
    return _check(lib().optiml_cross_entropy(N, Cn, _addr(logits), ld, _addr(labels), _addr(loss), _stream(stream)))


def optiml_layernorm(rows, length, x, y, eps, stream=None):
    return _check(lib().optiml_layernorm(rows, length, _addr(x), _addr(y), eps, _stream(stream)))


def optiml_mhsa(batch, N, d_model, heads, Q, K, V, O, dtype, stream=None):
    return _check(lib().optiml_mhsa(batch, N, d_model, heads, _addr(Q), _addr(K), _addr(V), _addr(O), dtype,
                                    _stream(stream)))


def optiml_transpose(rows, cols, src, ld_src, dst, ld_dst, elem_bytes, stream=None):
    return _check(lib().optiml_transpose(rows, cols, _addr(src), ld_src, _addr(dst), ld_dst, elem_bytes, _stream(stream)))


def optiml_gemm_cross_entropy(M, N, K, A, lda, B, ldb, bias, labels, loss, layout, dtype, stream=None):
    return _check(lib().optiml_gemm_cross_entropy(M, N, K, _addr(A), lda, _addr(B), ldb, _addr(bias), _addr(labels),
                                                  _addr(loss), layout, dtype, _stream(stream)))


def optiml_gemm_cross_entropy_rows(M, N, K, A, lda, B, ldb, bias, labels, row_loss, loss, layout, dtype, stream=None):
    return _check(lib().optiml_gemm_cross_entropy_rows(M, N, K, _addr(A), lda, _addr(B), ldb, _addr(bias), _addr(labels),
                                                       _addr(row_loss), _addr(loss), layout, dtype, _stream(stream)))


def optiml_gemm_layernorm(M, N, K, A, lda, B, ldb, bias, Y, ldy, eps, layout, dtype, stream=None):
    return _check(lib().optiml_gemm_layernorm(M, N, K, _addr(A), lda, _addr(B), ldb, _addr(bias), _addr(Y), ldy, eps,
                                              layout, dtype, _stream(stream)))


def optiml_gemm_layernorm_path(M, N, K, A, lda, B, ldb, bias, Y, ldy, layout, dtype):
    return lib().optiml_gemm_layernorm_path(M, N, K, _addr(A), lda, _addr(B), ldb, _addr(bias), _addr(Y), ldy, layout, dtype)


def optiml_gemm_cross_entropy_path(M, N, K, A, lda, B, ldb, bias, layout, dtype):
    return lib().optiml_gemm_cross_entropy_path(M, N, K, _addr(A), lda, _addr(B), ldb, _addr(bias), layout, dtype)


def optiml_set_workspace(ptr, nbytes):
    """Caller-supplied workspace for the current device (None, 0: back to the library's own)."""
    return _check(lib().optiml_set_workspace(_addr(ptr), nbytes))


def optiml_workspace_bytes():
    return lib().optiml_workspace_bytes()


def optiml_gemm_epilogue_mx(M, N, K, A, lda, scaleA, lds_a, B, ldb, scaleB, lds_b, bias, C, ldc, dtype=4, act=0, stream=None):
    """Block-scaled E2M1 contraction (A [M][K], B [N][K], one E8M0 scale per 32 elements of k), bf16 result."""
    return _check(lib().optiml_gemm_epilogue_mx(M, N, K, _addr(A), lda, _addr(scaleA), lds_a, _addr(B), ldb, _addr(scaleB), lds_b,
                                                _addr(bias), _addr(C), ldc, dtype, act, _stream(stream)))


def optiml_gemm_epilogue_mx_path(M, N, K, A, lda, scaleA, lds_a, B, ldb, scaleB, lds_b, bias, C, ldc, dtype=4):
    return lib().optiml_gemm_epilogue_mx_path(M, N, K, _addr(A), lda, _addr(scaleA), lds_a, _addr(B), ldb, _addr(scaleB), lds_b,
                                              _addr(bias), _addr(C), ldc, dtype)


def optiml_set_wait_limit(clocks):
    """Bound, in shader clocks, of the wait between the workgroups of one long LayerNorm row."""
    lib().optiml_set_wait_limit(int(clocks))


def optiml_status_string(status):
    return lib().optiml_status_string(status).decode()


def optiml_last_hip_error():
    return lib().optiml_last_hip_error()


def variant_names():
    return [optiml_variant_name(i) for i in range(optiml_variant_count())]
