"""The C-ABI boundary on a machine without a GPU: the library loads, exports every
declared symbol, and every invalid-argument path answers before touching the GPU."""
import ctypes
import os
import re

import pytest

from paper_2602_12305_amd import binding as ob

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "optiml.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(optiml_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = ctypes.CDLL(ob.LIB_PATH)
    names = declared_symbols()
    assert len(names) == 30
    for n in names:
        assert hasattr(L, n), n
    assert sorted(ob.SIGNATURES) == names


def test_variant_table():
    n = ob.optiml_variant_count()
    names = ob.variant_names()
    assert n == len(names) >= 3 and len(set(names)) == n
    assert names[0].startswith("generic")
    assert ob.optiml_variant_name(-1) is None and ob.optiml_variant_name(n) is None
    assert any(s.startswith("skinny_f32") for s in names)
    for dt in ("f32", "bf16"):
        for lay in ("rr", "rc", "cr", "cc"):
            assert any(s.startswith(f"tile_{dt}_{lay}_") for s in names)


def test_status_strings():
    assert ob.optiml_status_string(0) == "ok"
    for s in (-1, -2, -3, 7):
        assert ob.optiml_status_string(s)
    assert ob.optiml_last_hip_error() == 0


P = 0x10000  # a fake, 16-byte aligned device address: never dereferenced on these paths


def call(batch=1, M=8, N=8, K=8, A=P, lda=8, sA=0, B=P, ldb=8, sB=0, bias=P, sBias=0, C=P, ldc=8, sC=0,
         layout=0, dtype=0, act=0):
    return ob.lib().optiml_gemm_epilogue_strided_batched(batch, M, N, K, A, lda, sA, B, ldb, sB, bias, sBias,
                                                         C, ldc, sC, layout, dtype, act, None)


@pytest.mark.parametrize("kw", [
    dict(M=-1), dict(N=-1), dict(K=-1), dict(batch=-1),
    dict(A=None), dict(B=None), dict(C=None),
    dict(lda=7), dict(ldb=7), dict(ldc=7),
    dict(layout=1, K=16, ldb=8), dict(layout=2, M=16, lda=8),
    dict(layout=8), dict(layout=-1), dict(layout=4, M=16, ldc=8), dict(dtype=8), dict(dtype=-1), dict(act=4), dict(act=-1),
    dict(sA=-1), dict(sB=-1), dict(sBias=-1), dict(sC=-1),
    dict(batch=2, sC=63), dict(batch=2, sC=0),
])
def test_invalid_arguments_are_rejected_on_the_host(kw):
    assert call(**kw) == ob.ERR_INVALID_ARG


@pytest.mark.parametrize("kw", [dict(M=0), dict(N=0), dict(batch=0), dict(M=0, A=None, C=None)])
def test_empty_problems_are_ok_without_a_gpu(kw):
    assert call(**kw) == ob.OK


def test_plain_and_ex_entry_points_validate_too():
    L = ob.lib()
    assert L.optiml_gemm_epilogue(8, 8, 8, P, 8, P, 8, None, None, 8, 0, 0, None) == ob.ERR_INVALID_ARG
    assert L.optiml_gemm_epilogue(8, 8, 8, P, 8, P, 4, None, P, 8, 0, 0, None) == ob.ERR_INVALID_ARG
    assert L.optiml_gemm_epilogue_ex(8, 8, 8, P, 8, P, 8, None, P, 8, 9, 0, 0, None) == ob.ERR_INVALID_ARG
    assert L.optiml_gemm_epilogue(0, 8, 8, None, 8, None, 8, None, None, 8, 0, 0, None) == ob.OK
    assert L.optiml_gemm_epilogue_variant(1, 8, 8, 8, P, 8, 0, P, 8, 0, None, 0, P, 8, 0, 0, 0, 0, None, 9999) == ob.ERR_INVALID_ARG
    with pytest.raises(ob.OptimlError):
        ob.optiml_gemm_epilogue(8, 8, 8, P, 8, P, 8, None, 0, 8, 0, 0, stream=0)


def test_streaming_entry_points_validate_on_the_host():
    L = ob.lib()
    assert L.optiml_elementwise(-1, P, P, 0, None) == ob.ERR_INVALID_ARG
    assert L.optiml_elementwise(8, P, P, 2, None) == ob.ERR_INVALID_ARG          # unknown op
    assert L.optiml_elementwise(8, None, P, 0, None) == ob.ERR_INVALID_ARG
    assert L.optiml_elementwise(8, P, None, 1, None) == ob.ERR_INVALID_ARG
    assert L.optiml_elementwise(0, None, None, 0, None) == ob.OK                   # nothing to do
    assert L.optiml_reduce(-1, P, P, 0, P, None) == ob.ERR_INVALID_ARG
    assert L.optiml_reduce(8, P, P, 3, P, None) == ob.ERR_INVALID_ARG
    assert L.optiml_reduce(8, P, P, 0, None, None) == ob.ERR_INVALID_ARG           # no place for the result
    assert L.optiml_reduce(8, None, None, 0, P, None) == ob.ERR_INVALID_ARG
    assert L.optiml_reduce(8, P, None, 1, P, None) == ob.ERR_INVALID_ARG           # the dot product reads y
    assert L.optiml_reduce(8, P, None, 2, P, None) == ob.ERR_INVALID_ARG


def test_row_wise_entry_points_validate_on_the_host():
    L = ob.lib()
    assert L.optiml_cross_entropy(-1, 8, P, 8, P, P, None) == ob.ERR_INVALID_ARG
    assert L.optiml_cross_entropy(4, 0, P, 8, P, P, None) == ob.ERR_INVALID_ARG       # no classes
    assert L.optiml_cross_entropy(4, 8, P, 7, P, P, None) == ob.ERR_INVALID_ARG       # ld shorter than a row
    assert L.optiml_cross_entropy(4, 8, P, 8, P, None, None) == ob.ERR_INVALID_ARG
    assert L.optiml_cross_entropy(4, 8, None, 8, P, P, None) == ob.ERR_INVALID_ARG
    assert L.optiml_cross_entropy(4, 8, P, 8, None, P, None) == ob.ERR_INVALID_ARG
    assert L.optiml_layernorm(-1, 8, P, P, 1e-5, None) == ob.ERR_INVALID_ARG
    assert L.optiml_layernorm(4, -8, P, P, 1e-5, None) == ob.ERR_INVALID_ARG
    assert L.optiml_layernorm(4, 8, P, P, -1.0, None) == ob.ERR_INVALID_ARG
    assert L.optiml_layernorm(4, 8, P, P, float("nan"), None) == ob.ERR_INVALID_ARG
    assert L.optiml_layernorm(4, 8, None, P, 1e-5, None) == ob.ERR_INVALID_ARG
    assert L.optiml_layernorm(4, 8, P, None, 1e-5, None) == ob.ERR_INVALID_ARG
    assert L.optiml_layernorm(0, 8, None, None, 1e-5, None) == ob.OK
    assert L.optiml_layernorm(4, 0, None, None, 1e-5, None) == ob.OK


def test_attention_entry_point_validates_on_the_host():
    L = ob.lib()
    ok = (1, 64, 256, 4, P, P, P, P, 1, None)
    bad = [(-1, 64, 256, 4, P, P, P, P, 1, None), (1, -64, 256, 4, P, P, P, P, 1, None), (1, 64, 0, 4, P, P, P, P, 1, None),
           (1, 64, 256, 0, P, P, P, P, 1, None), (1, 64, 256, 3, P, P, P, P, 1, None),       # 256 columns, 3 heads
           (1, 64, 256, 4, P, P, P, P, 3, None), (1, 64, 256, 4, None, P, P, P, 1, None),
           (1, 64, 256, 4, P, None, P, P, 1, None), (1, 64, 256, 4, P, P, None, P, 1, None), (1, 64, 256, 4, P, P, P, None, 1, None)]
    for args in bad:
        assert L.optiml_mhsa(*args) == ob.ERR_INVALID_ARG, args
    assert L.optiml_mhsa(0, 64, 256, 4, None, None, None, None, 1, None) == ob.OK
    assert L.optiml_mhsa(1, 0, 256, 4, None, None, None, None, 0, None) == ob.OK
    assert L.optiml_mhsa(1, 64, 1024, 2, P, P, P, P, 0, None) == ob.ERR_UNSUPPORTED           # d_k = 512
    del ok


def sel(batch, M, N, K, layout=0, dtype=0, A=P, lda=None, ldb=None, ldc=None, bias=P):
    a_col, b_col = (layout >> 1) & 1, layout & 1
    lda = lda if lda is not None else (M if a_col else K)
    ldb = ldb if ldb is not None else (K if b_col else N)
    ldc = ldc if ldc is not None else (M if layout & 4 else N)
    v = ob.optiml_select_variant(batch, M, N, K, A, lda, M * K, P, ldb, K * N, bias, N, P, ldc, M * N, layout, dtype, 0)
    return ob.optiml_variant_name(v) if v >= 0 else v


def test_dispatch_by_shape_dtype_layout_alignment():
    assert sel(1, 16, 16384, 16384) == "skinny_f32_dma_wk4_cg2_ns2_nt1"               # B read once, straight to LDS
    assert sel(1, 8, 4096, 4096).startswith("skinny_f32")
    assert sel(1, 4096, 4096, 4096, layout=1).startswith("ring_f32_rc_128x128")
    assert sel(1, 8192, 8192, 8192, dtype=1).startswith("ring_bf16_rr_256x256")
    assert sel(32, 2048, 2048, 512, dtype=1).startswith("ring_bf16_rr_128x256_w1x4")   # many short tiles: two workgroups to a CU
    assert sel(1, 8192, 8192, 8192, dtype=2).startswith("ring_f16_rr_256x256")      # binary16: the same kernels
    assert sel(32, 2048, 2048, 512, dtype=2, layout=1).startswith("ring_f16_rc_128x256_w1x4")
    assert sel(1, 1024, 1024, 64, layout=2, dtype=2).startswith("tile_f16_cr_")
    assert sel(1, 1000, 1001, 64, dtype=2) == "generic_64x64"
    assert sel(1, 8192, 8192, 8192, layout=2, dtype=1) == "xa_ring"       # column-major A: row-major copy, then a ring kernel
    assert sel(1, 4096, 4096, 4096, layout=3) == "xa_ring"
    assert sel(1, 64, 64, 64, layout=2, dtype=1).startswith("tile_bf16_cr_")        # too little work to pay for the copy
    assert sel(1, 64, 4096, 4096, layout=2, dtype=1) == "xa_ring"                   # ... a few rows: copied, then streamed
    assert sel(1, 16, 16384, 16384, dtype=1).startswith("skinny_bf16_wn1_wk4_cg2")     # 16-bit storage streams B the same way
    assert sel(1, 16, 8192, 8192, dtype=1) == "skinny_bf16_dma_wk4_cg1_ns4_nt0"           # a smaller B: straight to LDS, 128 columns a workgroup
    assert sel(1, 7, 4096, 4096, dtype=2).startswith("skinny_f16_dma_wk4_cg1")        # a small B: 128 columns a workgroup
    assert sel(1, 8, 4096, 4096).startswith("skinny_f32_dma_wk4_cg1") and sel(1, 8, 4096, 4096, layout=1, dtype=1).startswith("skinnyrc_bf16_dma_wk4_cg2")
    assert "nt0" in sel(1, 32, 16384, 1024, dtype=1)                                   # two blocks of rows: B is left in the caches
    assert sel(1, 32, 16384, 16384, dtype=1).startswith("skinny_bf16")                # two blocks of rows still beat one row of tiles
    assert not sel(1, 64, 32768, 4096, dtype=1).startswith("skinny")                 # ... but not with a short K
    assert not sel(1, 256, 16384, 16384, dtype=1).startswith("skinny")
    # column-major C (layout + 4): the transposed problem, served by kernels that take a bias down the rows
    assert sel(1, 8192, 8192, 8192, layout=4 + 1, dtype=1).startswith("ring_bf16_rc_256x256")   # B^T row-major, A^T column-major
    assert sel(1, 8192, 8192, 8192, layout=4 + 0, dtype=1) == "xa_ring"                          # B^T column-major: copied
    assert sel(1, 4096, 4096, 4096, layout=4 + 3).startswith("ring_f32_rr")
    assert sel(32, 2048, 2048, 512, layout=4 + 1, dtype=1).startswith("ring_bf16_rc")            # not the persistent kernel
    assert sel(1, 16, 16384, 16384, layout=4 + 3).startswith("skinny_f32")                       # 16 columns of C^T: streamed, bias down the rows
    assert sel(1, 16384, 16, 16384, layout=4 + 3).startswith("skinny_f32") and sel(1, 4096, 8, 4096, layout=4 + 1, dtype=1).startswith("skinnyrc_bf16")
    assert sel(1, 8192, 8192, 8192, layout=1, dtype=3).startswith("ring_f8_rc_256x256")          # E4M3, k contiguous in both
    assert sel(1, 8192, 8192, 8192, layout=0, dtype=3) == "xk_ring_f8"                            # ... otherwise copied that way
    assert sel(1, 100, 100, 100, layout=0, dtype=3) == "generic_64x64"
    assert sel(1, 16, 16384, 16384, layout=1).startswith("skinnyrc_f32_dma_wk4_cg4_ns2")                # column-major B: streamed too
    assert sel(1, 32, 16384, 16384, layout=1, dtype=1).startswith("skinnyrc_bf16") and not sel(1, 512, 16384, 16384, layout=1, dtype=1).startswith("skinny")
    # by estimated time: a few blocks of rows streamed, then the smallest tiles that waste no rows
    assert sel(1, 64, 4096, 4096, layout=1, dtype=1).startswith("skinnyrc_bf16") and sel(1, 64, 4096, 4096, layout=1).startswith("skinnyrc_f32")
    assert sel(1, 128, 8192, 8192, layout=1, dtype=1).startswith("direct_bf16_rc_128x128")
    assert sel(1, 2048, 2048, 2048, dtype=1).startswith("direct_bf16_rr_128x128") and sel(1, 4096, 4096, 4096, dtype=1).startswith("ring_bf16_rr_256x256")
    assert sel(1, 4096, 512, 4096).startswith("skinny_f32") and sel(1, 512, 8192, 256).startswith("ring_f32_rr_128x128")
    assert sel(1, 16, 16384, 16384, layout=1, dtype=1).startswith("skinnyrc_bf16") and sel(1, 3, 4096, 4096, layout=1, dtype=3).startswith("skinnyrc_f8")
    assert sel(1, 256, 256, 256).startswith("skinny_f32_dma_wk8_cg1")                          # small: streamed per 16 rows, eight waves deep in k
    assert "nt0" in sel(1, 512, 2048, 2048) and sel(1, 512, 2048, 2048).startswith("skinny_f32_dma")   # many blocks of rows: B is left in the caches
    assert sel(1, 1024, 1024, 1024).startswith("skinny_f32")
    assert sel(1, 2048, 2048, 2048).startswith("ring_f32_rr")          # re-reading B no longer pays
    assert sel(1, 256, 256, 256, layout=2) == "xa_ring"                       # copied, then streamed like the row-major problem
    assert sel(1, 1024, 1024, 64, layout=3, dtype=1).startswith("tile_bf16_cc_")
    # K = 0, misaligned base, odd leading dimension, ragged contiguous extent -> guarded fallback
    assert sel(1, 64, 64, 0).startswith("generic")
    assert sel(1, 64, 64, 64, A=P + 4).startswith("generic") and sel(1, 100, 100, 52, lda=53).startswith("generic")
    assert sel(1, 512, 512, 512, A=P + 4) == "xpad" and sel(1, 512, 512, 512, lda=513) == "xpad"   # worth the copies already
    assert sel(1, 512, 510, 512, ldb=512, ldc=512) in ("generic_64x64", "xpad")  # N % 4 != 0 with row-major B
    # ... and when the problem is large enough to pay for copies into an aligned, padded form: those, then a fast kernel
    assert sel(1, 4096, 4096, 4096, A=P + 4, dtype=1) == "xpad" and sel(1, 4097, 4097, 4097, dtype=1) == "xpad"
    assert sel(1, 2048, 2050, 2048, dtype=2) == "xpad" and sel(1, 3001, 3001, 3001, layout=3) == "xpad"
    assert sel(1, 512, 510, 512, layout=1, ldc=512).startswith("skinnyrc_f32")  # fine when k is contiguous
    assert sel(1, 16, 1024, 1022, lda=1024) in ("generic_64x64", "xpad")
    assert sel(1, 16, 1024, 1024, dtype=1).startswith("skinny_bf16")
    assert sel(1, 8, 8, 8, layout=8) == ob.ERR_INVALID_ARG


def test_variant_supports_is_host_only_and_consistent():
    names = ob.variant_names()
    args = (1, 16, 1024, 1024, P, 1024, 0, P, 1024, 0, P, 0, P, 1024, 0, 0, 0, 0)
    ok = [n for i, n in enumerate(names) if ob.optiml_variant_supports(i, *args) == ob.OK]
    assert any(n.startswith("generic") for n in ok) and any(n.startswith("skinny") for n in ok)
    assert all(not n.startswith("tile_bf16") for n in ok) and all("_rc_" not in n for n in ok)
    assert ob.optiml_variant_supports(len(names), *args) == ob.ERR_INVALID_ARG
    bf16 = (1, 16, 1024, 1024, P, 1024, 0, P, 1024, 0, P, 0, P, 1024, 0, 0, 1, 0)
    sk = next(i for i, n in enumerate(names) if n.startswith("skinny"))
    assert ob.optiml_variant_supports(sk, *bf16) == ob.ERR_UNSUPPORTED
    assert ob.lib().optiml_gemm_epilogue_variant(*bf16, None, sk) == ob.ERR_UNSUPPORTED


def test_fused_cross_entropy_entry_point_validates_and_picks_its_kernel_on_the_host():
    L = ob.lib()
    #       M   N    K    A  lda  B  ldb bias labels loss layout dtype stream
    bad = [(-1, 64, 128, P, 128, P, 64, P, P, P, 0, 1, None), (8, 0, 128, P, 128, P, 64, P, P, P, 0, 1, None),
           (8, 64, -1, P, 128, P, 64, P, P, P, 0, 1, None), (8, 64, 128, P, 128, P, 64, P, P, None, 0, 1, None),
           (8, 64, 128, P, 128, P, 64, P, None, P, 0, 1, None), (8, 64, 128, None, 128, P, 64, P, P, P, 0, 1, None),
           (8, 64, 128, P, 128, None, 64, P, P, P, 0, 1, None), (8, 64, 128, P, 127, P, 64, P, P, P, 0, 1, None),
           (8, 64, 128, P, 128, P, 63, P, P, P, 0, 1, None), (8, 64, 128, P, 128, P, 127, P, P, P, 1, 1, None),
           (8, 64, 128, P, 7, P, 64, P, P, P, 2, 1, None), (8, 64, 128, P, 128, P, 64, P, P, P, 4, 1, None),
           (8, 64, 128, P, 128, P, 64, P, P, P, 0, 3, None)]
    for args in bad:
        assert L.optiml_gemm_cross_entropy(*args) == ob.ERR_INVALID_ARG, args
    path = lambda M, N, K, layout, dtype, A=P, lda=None, ldb=None: L.optiml_gemm_cross_entropy_path(
        M, N, K, A, lda if lda is not None else (M if layout & 2 else K), P, ldb if ldb is not None else (K if layout & 1 else N),
        P, layout, dtype)
    assert path(8192, 32768, 4096, 0, 1) == 0 and path(8192, 32768, 4096, 1, 2) == 0     # 16-bit, A row-major: matrix pipe
    assert path(300, 515, 160, 1, 1) == 0                                                  # ragged N with a column-major B
    assert path(300, 516, 160, 0, 1) == 1                                                  # row-major B rows not whole chunks
    assert path(8192, 32768, 4096, 0, 0) == 0 and path(100, 130, 64, 1, 0) == 0            # fp32: its own ring kernel
    assert path(100, 130, 48, 1, 0) == 1 and path(100, 130, 64, 0, 0) == 1                 # K < 64; row-major B rows not whole chunks
    assert path(8192, 32768, 4096, 2, 1) == 1                                              # A column-major
    assert path(64, 64, 96, 0, 1) == 1 and path(64, 64, 0, 0, 1) == 1                     # K too short for the ring, K = 0
    assert path(64, 64, 128, 0, 1, A=P + 2) == 1                                           # misaligned A
    assert path(8, 64, 128, 0, 5) == ob.ERR_INVALID_ARG


def test_transpose_entry_point_validates_on_the_host():
    L = ob.lib()
    bad = [(-1, 8, P, 8, P, 8, 4, None), (8, -1, P, 8, P, 8, 4, None), (8, 8, P, 7, P, 8, 4, None), (8, 8, P, 8, P, 7, 4, None),
           (8, 8, P, 8, P, 8, 3, None), (8, 8, P, 8, P, 8, 8, None), (8, 8, None, 8, P, 8, 4, None), (8, 8, P, 8, None, 8, 2, None)]
    for args in bad:
        assert L.optiml_transpose(*args) == ob.ERR_INVALID_ARG, args
    assert L.optiml_transpose(0, 8, None, 8, None, 0, 4, None) == ob.OK
    assert L.optiml_transpose(8, 0, None, 0, None, 8, 2, None) == ob.OK


def test_operand_spans_that_would_overflow_are_rejected_on_the_host():
    big = 1 << 46
    # (M - 1) * ldc + N, (batch - 1) * stride and the operands' own spans all stay below 2^47 elements
    assert call(M=4, ldc=big, sC=0) == ob.ERR_INVALID_ARG
    assert call(M=1 << 40, lda=1 << 40, K=8) == ob.ERR_INVALID_ARG
    assert call(batch=4, sA=big, sC=64) == ob.ERR_INVALID_ARG
    assert call(batch=1 << 62, sC=1 << 62) == ob.ERR_INVALID_ARG
    assert call(K=1 << 50, lda=1 << 50, ldb=8) == ob.ERR_INVALID_ARG
    L = ob.lib()
    assert L.optiml_gemm_cross_entropy(1 << 30, 8, 1 << 30, P, 1 << 30, P, 8, None, P, P, 0, 0, None) == ob.ERR_INVALID_ARG


def test_set_workspace_validates_on_the_host():
    L = ob.lib()
    assert L.optiml_set_workspace(P, -1) == ob.ERR_INVALID_ARG
    assert L.optiml_set_workspace(None, 4096) == ob.ERR_INVALID_ARG
    assert L.optiml_set_workspace(P, 0) == ob.ERR_INVALID_ARG
    assert L.optiml_set_workspace(P + 16, 4096) == ob.ERR_INVALID_ARG      # not 256-byte aligned


def test_mfma_probe_validates_on_the_host():
    L = ob.lib()
    assert L.optiml_mfma_probe(P, 1 << 30, P, 1 << 30, -1, 1, 0, None, None) == ob.ERR_INVALID_ARG
    assert L.optiml_mfma_probe(P, 1 << 30, P, 1 << 30, 10, 0, 0, None, None) == ob.ERR_INVALID_ARG     # fp32: not offered
    assert L.optiml_mfma_probe(P, 1 << 30, P, 1 << 30, 10, 1, 7, None, None) == ob.ERR_INVALID_ARG     # 0, 8, 12 or 16
    assert L.optiml_mfma_probe(None, 1 << 30, P, 1 << 30, 10, 1, 0, None, None) == ob.ERR_INVALID_ARG
    assert L.optiml_mfma_probe(P + 8, 1 << 30, P, 1 << 30, 10, 1, 0, None, None) == ob.ERR_INVALID_ARG


def test_fused_layernorm_entry_point_validates_and_picks_its_kernel_on_the_host():
    L = ob.lib()
    ok = dict(M=512, N=768, K=256, A=P, lda=256, B=P, ldb=768, bias=P, Y=P, ldy=768, eps=1e-5, layout=0, dtype=1)

    def call_ln(**kw):
        a = dict(ok, **kw)
        return L.optiml_gemm_layernorm(a["M"], a["N"], a["K"], a["A"], a["lda"], a["B"], a["ldb"], a["bias"], a["Y"], a["ldy"],
                                       a["eps"], a["layout"], a["dtype"], None)

    def path(**kw):
        a = dict(ok, **kw)
        return L.optiml_gemm_layernorm_path(a["M"], a["N"], a["K"], a["A"], a["lda"], a["B"], a["ldb"], a["bias"], a["Y"],
                                            a["ldy"], a["layout"], a["dtype"])

    for bad in (dict(M=-1), dict(N=-1), dict(K=-1), dict(ldy=767), dict(lda=255), dict(ldb=767), dict(Y=None), dict(A=None),
                dict(B=None), dict(eps=-1.0), dict(eps=float("nan")), dict(layout=4), dict(dtype=3), dict(dtype=9)):
        assert call_ln(**bad) == ob.ERR_INVALID_ARG, bad
    assert call_ln(M=0) == ob.OK and call_ln(N=0, ldb=0, ldy=0) == ob.OK           # nothing to write
    assert path() == 0 and path(dtype=0) == 0 and path(dtype=2, layout=1, ldb=256) == 0
    assert path(layout=2, lda=512) == 1                         # column-major A
    assert path(K=0) == 1 and path(K=40, lda=40) == 1           # nothing to contract / too short for the ring
    assert path(A=P + 2) == 1                                   # misaligned operand
    assert path(dtype=0, Y=P + 4) == 1 and path(dtype=0, ldy=770) == 1   # fp32: z is written into Y with 16-byte stores
    assert path(dtype=1, Y=P + 2, ldy=771) == 0                 # 16-bit: z goes to the workspace, Y may sit anywhere


def test_e2m1_operands_are_validated_and_dispatched_before_any_gpu_call():
    """4-bit operands: two elements a byte along k, so K, lda, ldb (in elements) must be even and k contiguous in both."""
    ERR_INVALID, ERR_UNSUPPORTED = -1, -2
    assert ob.optiml_status_string(ERR_INVALID) and ob.optiml_status_string(ERR_UNSUPPORTED)
    assert sel(1, 8192, 8192, 8192, layout=1, dtype=4).startswith("ring_f4_rc_256x256")
    assert sel(1, 16, 16384, 16384, layout=1, dtype=4).startswith("skinnyrc_f4")
    assert sel(1, 100, 100, 70, layout=1, dtype=4) == "generic_64x64"                   # 35 bytes of k a row
    assert sel(1, 512, 512, 512, layout=5, dtype=4) != ERR_UNSUPPORTED                   # column-major C of an RC problem: its mirror image
    for layout in (0, 2, 3, 4, 6, 7):
        assert sel(1, 512, 512, 512, layout=layout, dtype=4) == ERR_UNSUPPORTED
    assert sel(1, 512, 512, 511, layout=1, dtype=4) == ERR_INVALID                       # odd K
    assert sel(1, 512, 512, 512, layout=1, dtype=4, lda=513) == ERR_INVALID              # odd pitch
    assert sel(1, 512, 512, 512, layout=1, dtype=4, ldb=515) == ERR_INVALID
    assert sel(1, 512, 512, 512, layout=1, dtype=4, lda=510) == ERR_INVALID              # pitch shorter than a row
    assert sel(1, 512, 512, 512, layout=1, dtype=8) == ERR_INVALID                       # no such storage type
    assert sel(1, 8192, 8192, 8192, layout=1, dtype=5).startswith("ring_bf8_rc_256x256") and sel(1, 16, 16384, 16384, layout=1, dtype=5).startswith("skinnyrc_bf8")   # E5M2: the E4M3 kernels with the other format code
    assert sel(1, 8192, 8192, 8192, layout=0, dtype=5) == "xk_ring_f8" and sel(1, 100, 100, 100, layout=0, dtype=5) == "generic_64x64"


def test_six_bit_operands_are_validated_and_dispatched_before_any_gpu_call():
    """6-bit operands: a dense stream of 6-bit codes, so every row has to start on a byte (pitches and batch strides in
    elements, multiples of 4); the matrix-pipe path takes k contiguous in both operands, the fallback every layout."""
    ERR_INVALID = -1
    for dtype, tag in ((6, "f6"), (7, "bf6")):
        assert sel(1, 8192, 8192, 8192, layout=1, dtype=dtype) == f"xs_ring_{tag}_rc_256x256_w2x4_ns5_k64"
        assert sel(1, 300, 520, 228, layout=1, dtype=dtype).startswith("xs_ring_" + tag)   # any K that is a multiple of 4
        assert sel(1, 300, 520, 230, layout=1, dtype=dtype, lda=232, ldb=232) == "generic_64x64"
        assert sel(1, 33, 65, 8, layout=1, dtype=dtype) == "generic_64x64"                  # too little work to copy for
        assert sel(1, 300, 520, 100, layout=1, dtype=dtype) == "generic_64x64"
        assert sel(1, 512, 512, 512, layout=5, dtype=dtype).startswith("xs_ring_" + tag)   # column-major C: the mirror image
        for layout in (0, 2, 3, 4, 6, 7):
            assert sel(1, 512, 512, 512, layout=layout, dtype=dtype) == "generic_64x64"
        assert sel(1, 512, 512, 512, layout=1, dtype=dtype, lda=514) == ERR_INVALID        # a row would start inside a byte
        assert sel(1, 512, 512, 512, layout=1, dtype=dtype, ldb=513) == ERR_INVALID
        assert sel(1, 512, 512, 512, layout=1, dtype=dtype, lda=508) == ERR_INVALID        # pitch shorter than a row
        # no other kernel claims the storage type
        args = (1, 512, 512, 512, P, 512, 0, P, 512, 0, P, 0, P, 512, 0, 1, dtype, 0)
        takers = [ob.optiml_variant_name(v) for v in range(ob.optiml_variant_count()) if ob.optiml_variant_supports(v, *args) == ob.OK]
        assert takers == ["generic_64x64", f"xs_ring_{tag}_rc_256x256_w2x4_ns5_k64"]


def test_block_scaled_entry_point_validates_and_picks_its_kernel_on_the_host():
    L = ob.lib()
    def call(M=512, N=512, K=512, A=P, lda=None, sA=P, lds_a=None, B=P, ldb=None, sB=P, lds_b=None, bias=P, C=P, ldc=None, dtype=4, act=0):
        lda = K if lda is None else lda; ldb = K if ldb is None else ldb; ldc = N if ldc is None else ldc
        lds_a = K // 32 if lds_a is None else lds_a; lds_b = K // 32 if lds_b is None else lds_b
        return (L.optiml_gemm_epilogue_mx(M, N, K, A, lda, sA, lds_a, B, ldb, sB, lds_b, bias, C, ldc, dtype, act, None),
                L.optiml_gemm_epilogue_mx_path(M, N, K, A, lda, sA, lds_a, B, ldb, sB, lds_b, bias, C, ldc, dtype))
    for kw in (dict(M=-1), dict(K=-32), dict(K=48), dict(lda=510), dict(lda=513), dict(ldb=511), dict(lds_a=15), dict(lds_b=3), dict(ldc=511),
               dict(dtype=8), dict(dtype=2), dict(dtype=1), dict(A=None), dict(B=None), dict(sA=None), dict(sB=None), dict(C=None)):
        assert call(**kw)[1] == ob.ERR_INVALID_ARG, kw
    assert call(act=7)[0] == ob.ERR_INVALID_ARG
    assert call(M=0, A=None, C=None)[0] == ob.OK and call(N=0)[0] == ob.OK                # nothing to do
    assert call()[1] == 0 and call(M=4096, N=4096, K=4096)[1] == 0                        # the matrix-pipe tile kernel
    assert call(K=480)[1] == 1 and call(M=100, N=100)[1] == 1                             # K not whole k-tiles; a small C
    assert call(M=16, N=4096, K=1024)[1] == 2 and call(M=128, N=1024)[1] == 2 and call(M=129, N=1024)[1] == 0   # few rows of E2M1: streamed
    assert call(M=48, N=16384, K=16384)[1] == 2 and call(M=49, N=16384, K=16384)[1] == 0 and call(M=128, N=8192, K=8192)[1] == 2   # more than three blocks of rows: only over a B the Infinity Cache holds
    assert call(M=16, N=4096, K=1056)[1] == 1 and call(M=16, N=4096, dtype=3)[1] == 0   # (other element types: the tile kernel)
    assert call(A=P + 2)[1] == 1                                                          # an address the wide loads cannot take
    assert call(sA=P + 1)[1] == 0 and call(lds_a=18)[1] == 0                              # the scales are copied first: any address and pitch
    assert call(lda=514)[1] == 1
    assert call(dtype=3)[1] == 0 and call(dtype=5)[1] == 0 and call(dtype=3, K=320)[1] == 0      # 8-bit elements: k-tiles of 64
    assert call(dtype=3, K=480)[1] == 1 and call(dtype=5, K=192)[1] == 1 and call(dtype=3, lda=513)[1] == 1   # (odd pitches are valid there)
    # 6-bit elements: copied into 32-byte slots first, so any address and any pitch that is a multiple of 4 elements
    assert call(dtype=6)[1] == 0 and call(dtype=7, K=320)[1] == 0 and call(dtype=6, A=P + 3, lda=516)[1] == 0
    assert call(dtype=6, K=480)[1] == 1 and call(dtype=7, K=192)[1] == 1 and call(dtype=7, M=100, N=100)[1] == 1
    assert call(dtype=6, lda=514)[1] == ob.ERR_INVALID_ARG and call(dtype=7, ldb=513)[1] == ob.ERR_INVALID_ARG
