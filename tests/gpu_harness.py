"""Run the HIP library on host arrays and compare with the CPU oracle (GPU tests only)."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from inputs import synth
from paper_2602_12305_amd import binding
from helpers import e1, store

# binary16: one rounding of the output, half a step = 2^-12 .. 2^-11 relative across a binade (4.9e-4 at most),
# plus fp32 accumulation: bar 1e-3
TOL = {synth.DTYPE_F32: 1e-5, synth.DTYPE_BF16: 2e-2, synth.DTYPE_F16: 1e-3, synth.DTYPE_F8E4M3: 2e-2,
       synth.DTYPE_F4E2M1: 2e-2, synth.DTYPE_F8E5M2: 2e-2, synth.DTYPE_F6E2M3: 2e-2, synth.DTYPE_F6E3M2: 2e-2}     # 8-, 6- and 4-bit operands: bf16 result


def c_dtype(dtype):
    """Storage type of C for a contraction dtype (8-bit and 4-bit operands give a bf16 result)."""
    return synth.DTYPE_BF16 if dtype in (synth.DTYPE_F8E4M3, synth.DTYPE_F4E2M1, synth.DTYPE_F8E5M2, synth.DTYPE_F6E2M3, synth.DTYPE_F6E3M2) else dtype


def ld_elements(X, dtype):
    """Leading dimension, in elements, of a storage array (E2M1 arrays hold two elements a byte, 6-bit arrays four in three)."""
    if dtype in (synth.DTYPE_F6E2M3, synth.DTYPE_F6E3M2):
        return X.shape[-1] * 4 // 3
    return X.shape[-1] * (2 if dtype == synth.DTYPE_F4E2M1 else 1)
POISON = 12345.0


def to_dev(x: np.ndarray | None):
    if x is None:
        return None
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).cuda()
    return torch.from_numpy(x).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    a = t.cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.int16 else a


def alloc_c(batch, M, ldc, dtype, fill=POISON):
    """C storage [batch, M, ldc], pre-filled so that untouched entries (padding) can be checked."""
    dtype = c_dtype(dtype)
    if dtype == synth.DTYPE_F32:
        return torch.full((batch, M, ldc), fill, dtype=torch.float32, device="cuda")
    bits = int(synth.to_bits(np.array([fill], dtype=np.float32), dtype)[0])
    return torch.full((batch, M, ldc), np.int16(np.uint16(bits).view(np.int16)).item(), dtype=torch.int16, device="cuda")


def c_values(Cd, dtype, N):
    """Device C storage -> (fp64 values [batch, M, N], padding region as fp32)."""
    h = to_host(Cd)
    f = synth.from_bits(h, c_dtype(dtype))
    return f[..., :N].astype(np.float64), f[..., N:]


def run_gpu(As, Bs, bias, batch, M, N, K, dtype, act, layout, *, ldc=None, variant=None,
            strideA=None, strideB=None, strideBias=None, entry="batched"):
    """As/Bs: storage arrays ([batch,] rows, ld).  Returns (Y fp64 [batch,M,N], pad region, device C)."""
    lda, ldb = ld_elements(As, dtype), ld_elements(Bs, dtype)
    c_col = bool(layout & 4)                       # column-major C: storage [batch, N, ldc >= M]
    crows, ccols = (N, M) if c_col else (M, N)
    ldc = ccols if ldc is None else ldc
    if strideA is None:
        strideA = As.shape[-2] * lda if batch > 1 else 0
    if strideB is None:
        strideB = Bs.shape[-2] * ldb if batch > 1 else 0
    if strideBias is None:
        strideBias = N if (bias is not None and batch > 1 and bias.size >= batch * N) else 0
    Ad, Bd, bd = to_dev(As), to_dev(Bs), to_dev(None if bias is None else np.ascontiguousarray(bias, dtype=np.float32))
    Cd = alloc_c(batch, crows, ldc, dtype)
    strideC = crows * ldc
    if variant is not None:
        binding.optiml_gemm_epilogue_variant(batch, M, N, K, Ad, lda, strideA, Bd, ldb, strideB, bd, strideBias,
                                             Cd, ldc, strideC, layout, dtype, act, variant)
    elif entry == "plain":
        assert batch == 1 and layout == 0
        binding.optiml_gemm_epilogue(M, N, K, Ad, lda, Bd, ldb, bd, Cd, ldc, dtype, act)
    elif entry == "ex":
        assert batch == 1
        binding.optiml_gemm_epilogue_ex(M, N, K, Ad, lda, Bd, ldb, bd, Cd, ldc, layout, dtype, act)
    else:
        binding.optiml_gemm_epilogue_strided_batched(batch, M, N, K, Ad, lda, strideA, Bd, ldb, strideB, bd,
                                                     strideBias, Cd, ldc, strideC, layout, dtype, act)
    torch.cuda.synchronize()
    Y, pad = c_values(Cd, dtype, ccols)
    if c_col:
        Y = np.ascontiguousarray(np.swapaxes(Y, -1, -2))
    return Y, pad, Cd


def check_against_oracle(A, B, bias, *, dtype, act, layout, pad=0, ldc_pad=0, variant=None, entry="batched",
                         exact=False, tol=None):
    """A [.., M, K], B [.., K, N] logical fp32 arrays.  Element-by-element comparison with the oracle:
    E1 within the dtype's tolerance, or exact equality (after the oracle's own bf16 rounding) when
    `exact`.  Also checks that padding columns of C were left alone."""
    batch = A.shape[0] if A.ndim == 3 else 1
    M, K = A.shape[-2:]; N = B.shape[-1]
    As = store(A, dtype, (layout >> 1) & 1, pad); Bs = store(B, dtype, layout & 1, pad)
    Y, padregion, _ = run_gpu(As, Bs, bias, batch, M, N, K, dtype, act, layout, ldc=(M if layout & 4 else N) + ldc_pad,
                              variant=variant, entry=entry)
    ref = oracle.gemm_epilogue(As, Bs, bias, M, N, K, dtype=dtype, act=act, layout=layout & 3, batch=batch)
    assert Y.shape == ref.shape
    if padregion.size:
        assert np.all(padregion == np.float32(POISON) if dtype == synth.DTYPE_F32 else
                      np.all(synth.to_bits(padregion, c_dtype(dtype)) == synth.to_bits(np.array([POISON], dtype=np.float32), c_dtype(dtype))[0]))
    if exact:
        if c_dtype(dtype) == synth.DTYPE_BF16:
            want = synth.bf16_bits_to_f32(oracle.bf16_from_double(ref)).astype(np.float64)
        elif dtype == synth.DTYPE_F16:
            want = oracle.f16_to_double(oracle.f16_from_double(ref))
        else:
            want = ref
        bad = np.argwhere(Y != want)
        assert bad.size == 0, f"{len(bad)} mismatches, first at {bad[0]}: got {Y[tuple(bad[0])]} want {want[tuple(bad[0])]}"
        return 0.0
    err = e1(Y, ref)
    limit = TOL[dtype] if tol is None else tol
    assert np.all(np.isfinite(Y)), "non-finite output"
    assert err <= limit, f"E1 = {err:.3e} > {limit:.1e}"
    return err
