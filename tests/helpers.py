"""Shared test utilities: exact rational evaluation on tiny shapes, storage helpers,
and the pass/fail error metric.  Nothing here is used by the product."""
from __future__ import annotations

from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np

from inputs import synth

getcontext().prec = 60


def store(X, dtype, col_major=False, pad=0):
    """Logical fp32 matrix (or [batch, r, c] stack) -> storage array [.., rows, ld] in the
    element type of `dtype`; `pad` extra elements per row hold a poison value."""
    X = np.asarray(X, dtype=np.float32)
    if col_major:
        X = np.swapaxes(X, -1, -2)
    X = np.ascontiguousarray(X)
    if pad:
        shp = X.shape[:-1] + (X.shape[-1] + pad,)
        P = np.full(shp, 777.0, dtype=np.float32)
        P[..., : X.shape[-1]] = X
        X = P
    return synth.to_bits(X, dtype)


def as_real(X, dtype):
    """Stored operand -> the exact real values it holds, as fp64."""
    if dtype != synth.DTYPE_F32:
        return synth.from_bits(X, dtype).astype(np.float64)
    return np.asarray(X, dtype=np.float64)


def exact_z(A, B, bias):
    """z[i][j] = bias[j] + sum_k a[i,k] b[k,j] in exact rational arithmetic (k descending,
    so the evaluation order differs from the oracle's)."""
    A = np.asarray(A, dtype=np.float64); B = np.asarray(B, dtype=np.float64)
    M, K = A.shape; N = B.shape[1]
    out = [[Fraction(0)] * N for _ in range(M)]
    for i in range(M):
        for j in range(N):
            s = Fraction(0)
            for k in range(K - 1, -1, -1):
                s += Fraction(float(A[i, k])) * Fraction(float(B[k, j]))
            if bias is not None:
                s += Fraction(float(bias[j]))
            out[i][j] = s
    return out


def _dec(fr: Fraction) -> Decimal:
    return Decimal(fr.numerator) / Decimal(fr.denominator)


def act_decimal(z, act) -> float:
    """Activation of an exact rational (or float) in 60-digit decimal arithmetic."""
    z = _dec(z) if isinstance(z, Fraction) else Decimal(float(z))
    if act == synth.ACT_NONE:
        return float(z)
    if act == synth.ACT_RELU:
        return float(z) if z > 0 else 0.0
    if act == synth.ACT_SILU:
        return float(z / (1 + (-z).exp()))
    if act == synth.ACT_GELU_TANH:
        pi = Decimal("3.14159265358979323846264338327950288419716939937510582097494")
        u = (Decimal(2) / pi).sqrt() * (z + Decimal("0.044715") * z * z * z)
        if u > 60:
            t = Decimal(1)
        elif u < -60:
            t = Decimal(-1)
        else:
            e = (2 * u).exp()
            t = (e - 1) / (e + 1)
        return float(Decimal("0.5") * z * (1 + t))
    raise ValueError(act)


def e1(y, y_ref):
    """max |y - y_ref| / max(|y_ref|, rho), rho = RMS of y_ref over the checked entries."""
    y = np.asarray(y, dtype=np.float64).ravel(); y_ref = np.asarray(y_ref, dtype=np.float64).ravel()
    if y_ref.size == 0:
        return 0.0
    rho = float(np.sqrt(np.mean(y_ref * y_ref)))
    den = np.maximum(np.abs(y_ref), rho if rho > 0 else 1.0)
    return float(np.max(np.abs(y - y_ref) / den))
