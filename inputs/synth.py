"""Seeded synthetic inputs for C = act(A.B + bias).

Counter-based generation: every element is a pure function of
(seed, tensor tag, batch, logical row, logical column), so storage order,
chunking and threading cannot change the data, and a column-major buffer
holds the same matrix as a row-major one.

This module holds no arithmetic of the operator itself (no products, sums,
bias or activation).  It is the only code the CPU checker and the GPU path
have in common: both read the host arrays made here.

The paper evaluates Matrix Multiplication (Table 4, task 2) on a task suite
whose sizes and inputs it does not print; the five workloads below are the
synthetic stand-ins, with the shapes and distributions fixed by the benchmark
configuration of this repository.
"""

from __future__ import annotations

import concurrent.futures as _cf
from dataclasses import dataclass, field

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_MAX_DIM = 1 << 24  # rows, cols < 2^24 ; batch < 2^16 (packed into one 64-bit counter)


def _mix64(x: np.ndarray) -> np.ndarray:
    """64-bit avalanche finaliser of SplitMix64 (Steele, Lea, Flood 2014)."""
    x = (x ^ (x >> np.uint64(30))) * _M1
    x = (x ^ (x >> np.uint64(27))) * _M2
    return x ^ (x >> np.uint64(31))


def _tag_hash(tag: str) -> np.uint64:
    """FNV-1a over the tag's bytes."""
    h = 0xCBF29CE484222325
    for byte in tag.encode("utf-8"):
        h = ((h ^ byte) * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    return np.uint64(h)


def _key(seed: int, tag: str, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        k = np.array([np.uint64(seed & 0xFFFFFFFFFFFFFFFF)], dtype=np.uint64)
        k = _mix64(k + _GOLDEN) ^ _tag_hash(tag)
        k = _mix64(k + np.uint64(stream + 1) * _GOLDEN)
    return k[0]


def _counters(batch: int, r0: int, r1: int, cols: int) -> np.ndarray:
    r = np.arange(r0, r1, dtype=np.uint64)[:, None]
    c = np.arange(cols, dtype=np.uint64)[None, :]
    return (np.uint64(batch) << np.uint64(48)) | (r << np.uint64(24)) | c


def _u01(key: np.uint64, ctr: np.ndarray) -> np.ndarray:
    """53-bit uniform in [0, 1) as fp64."""
    with np.errstate(over="ignore"):
        h = _mix64(key ^ _mix64(ctr * _GOLDEN + _GOLDEN))
    return (h >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def _fill(kind, seed, tag, batch, rows, cols, p0, p1, out):
    """out[batch, rows, cols] fp32 <- distribution `kind`, rounded once to fp32."""
    if rows >= _MAX_DIM or cols >= _MAX_DIM or batch >= (1 << 16):
        raise ValueError("dimension too large for the packed counter")
    k0, k1 = _key(seed, tag, 0), _key(seed, tag, 1)
    chunk = max(1, min(rows, (1 << 21) // max(cols, 1)))
    jobs = [(b, r0, min(rows, r0 + chunk)) for b in range(batch) for r0 in range(0, rows, chunk)]

    def work(job):
        b, r0, r1 = job
        ctr = _counters(b, r0, r1, cols)
        u = _u01(k0, ctr)
        if kind == "uniform":        # U[p0, p1)
            v = p0 + (p1 - p0) * u
        elif kind == "normal":       # N(p0, p1^2), Box-Muller, cosine branch only
            v = _u01(k1, ctr)
            v = p0 + p1 * np.sqrt(-2.0 * np.log1p(-u)) * np.cos(2.0 * np.pi * v)
        elif kind == "integers":     # integers in [p0, p1], each equally likely
            v = np.floor(p0 + (p1 - p0 + 1) * u)
        else:
            raise ValueError(kind)
        out[b, r0:r1, :] = v.astype(np.float32)

    if len(jobs) == 1:
        work(jobs[0])
    else:
        with _cf.ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(work, jobs))
    return out


def _gen(kind, seed, tag, rows, cols, p0, p1, batch=None):
    nb = 1 if batch is None else batch
    out = np.empty((nb, rows, cols), dtype=np.float32)
    _fill(kind, seed, tag, nb, rows, cols, p0, p1, out)
    return out[0] if batch is None else out


def uniform(seed, tag, rows, cols, lo=-1.0, hi=1.0, batch=None):
    """fp32 matrix (or [batch, rows, cols] stack) iid U[lo, hi)."""
    return _gen("uniform", seed, tag, rows, cols, float(lo), float(hi), batch)


def normal(seed, tag, rows, cols, mean=0.0, std=1.0, batch=None):
    """fp32 matrix iid N(mean, std^2)."""
    return _gen("normal", seed, tag, rows, cols, float(mean), float(std), batch)


def integers(seed, tag, rows, cols, lo=-3, hi=3, batch=None):
    """fp32 matrix of iid integers in [lo, hi] (exactly representable in bf16 for |v| <= 256)."""
    return _gen("integers", seed, tag, rows, cols, float(lo), float(hi), batch)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the uint16 bit patterns.
    NaN stays NaN (quiet bit forced), overflow rounds to infinity."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = ((u.astype(np.uint64) + np.uint64(0x7FFF) + lsb) >> np.uint64(16)).astype(np.uint16)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    return np.where(nan, ((u >> np.uint32(16)) | np.uint32(0x40)).astype(np.uint16), r)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to IEEE binary16 (nearest, ties to even; overflow to infinity); uint16 bit patterns."""
    with np.errstate(over="ignore"):
        return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def f16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(b, dtype=np.uint16).view(np.float16).astype(np.float32)


def f32_to_f8e4m3_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to OCP E4M3 (nearest, ties to even; magnitudes beyond 448 saturate to 448, NaN -> 0x7F); uint8."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    a = np.minimum(np.abs(np.nan_to_num(x.astype(np.float64), nan=0.0)), 448.0)
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -20)))
    e = np.maximum(e, -6.0)                              # below 2^-6 the spacing stays 2^-9 (subnormals)
    q = np.exp2(e - 3.0)                                 # spacing: 3 fraction bits
    r = np.rint(a / q) * q                               # numpy rounds half to even
    r = np.minimum(r, 448.0)
    ee = np.floor(np.log2(np.maximum(r, 2.0 ** -20)))
    normal = r >= 2.0 ** -6
    field = np.where(normal, ee + 7.0, 0.0)
    frac = np.where(normal, r / np.exp2(ee) * 8.0 - 8.0, r * 512.0)
    bits = (field.astype(np.int64) << 3 | frac.astype(np.int64)).astype(np.uint8)
    bits = np.where(np.isnan(x), np.uint8(0x7F), bits)
    return (bits | (np.signbit(x).astype(np.uint8) << 7)).astype(np.uint8)


def f8e4m3_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint8).astype(np.int64)
    e, f = (b >> 3) & 15, b & 7
    v = np.where(e == 0, f * 2.0 ** -9, (8 + f) * np.exp2(e - 10.0))
    v = np.where((e == 15) & (f == 7), np.nan, v)
    return np.where(b >> 7 == 1, -v, v).astype(np.float32)


def f32_to_f8e5m2_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to OCP E5M2 (nearest, ties to even; magnitudes that round beyond 57344 become infinity, as in
    binary16, of which E5M2 is the upper byte; NaN -> 0x7F); uint8."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    a = np.abs(np.nan_to_num(x.astype(np.float64), nan=0.0, posinf=1e300, neginf=-1e300))
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -40)))
    e = np.clip(e, -14.0, 15.0)                          # below 2^-14 the spacing stays 2^-16 (subnormals)
    q = np.exp2(e - 2.0)                                 # spacing: 2 fraction bits
    r = np.rint(np.minimum(a, 1e6) / q) * q              # numpy rounds half to even
    over = r > 57344.0                                   # 61440 is the first value that rounds up
    ee = np.floor(np.log2(np.maximum(r, 2.0 ** -40)))
    normal = r >= 2.0 ** -14
    field = np.where(normal, ee + 15.0, 0.0)
    frac = np.where(normal, r / np.exp2(ee) * 4.0 - 4.0, r * 65536.0)
    bits = (field.astype(np.int64) << 2 | frac.astype(np.int64)).astype(np.uint8)
    bits = np.where(over, np.uint8(0x7C), bits)
    bits = np.where(np.isnan(x), np.uint8(0x7F), bits)
    return (bits | (np.signbit(x).astype(np.uint8) << 7)).astype(np.uint8)


def f8e5m2_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """E5M2 is the upper byte of binary16."""
    b = np.ascontiguousarray(b, dtype=np.uint8).astype(np.uint16)
    return (b << 8).astype(np.uint16).view(np.float16).astype(np.float32)


# the eight magnitudes of OCP E2M1, by code
_F4_VALUES = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], dtype=np.float32)


def f32_to_f4e2m1_codes(x: np.ndarray) -> np.ndarray:
    """Nearest OCP E2M1 code of each fp32 value (ties to the even code, magnitudes beyond 6 saturate, NaN -> +0): uint8
    in 0..15, one code per element (not yet packed)."""
    x = np.nan_to_num(np.ascontiguousarray(x, dtype=np.float32), nan=0.0)
    a = np.minimum(np.abs(x), np.float32(6.0))
    # midpoints between neighbouring magnitudes; a tie goes to the even code (0, 1.0, 2.0, 4.0 have even codes)
    mids = (_F4_VALUES[:-1] + _F4_VALUES[1:]) / np.float32(2.0)
    code = np.searchsorted(mids, a, side="left").astype(np.int64)            # a == mid -> the lower code
    tie = np.isin(a, mids) & (code % 2 == 1)                                  # lower code odd -> take the upper, even one
    code = code + tie.astype(np.int64)
    return (code | (np.signbit(x).astype(np.int64) << 3)).astype(np.uint8)


def pack_f4(codes: np.ndarray) -> np.ndarray:
    """Two 4-bit codes to a byte along the last axis (even index in the low four bits); the last axis must be even."""
    c = np.ascontiguousarray(codes, dtype=np.uint8)
    if c.shape[-1] % 2:
        raise ValueError("an even number of 4-bit elements per row expected")
    return (c[..., 0::2] | (c[..., 1::2] << np.uint8(4))).astype(np.uint8)


def unpack_f4(packed: np.ndarray) -> np.ndarray:
    p = np.ascontiguousarray(packed, dtype=np.uint8)
    out = np.empty(p.shape[:-1] + (2 * p.shape[-1],), dtype=np.uint8)
    out[..., 0::2] = p & np.uint8(15)
    out[..., 1::2] = p >> np.uint8(4)
    return out


def f4e2m1_codes_to_f32(codes: np.ndarray) -> np.ndarray:
    c = np.ascontiguousarray(codes, dtype=np.uint8)
    v = _F4_VALUES[c & np.uint8(7)]
    return np.where((c >> np.uint8(3)) & np.uint8(1) == 1, -v, v).astype(np.float32)


# the 32 magnitudes of the OCP 6-bit types by code, written as runs of constant spacing: E2M3 (largest 7.5) has sixteen
# values 1/8 apart below 2 (eight subnormals, then the binade of 1), E3M2 (largest 28) eight values 1/16 apart below 1/2
_F6_VALUES = {
    6: np.concatenate([np.arange(0, 2, 0.125), np.arange(2, 4, 0.25), np.arange(4, 8, 0.5)]).astype(np.float32),
    7: np.concatenate([np.arange(0, 0.5, 0.0625), np.arange(0.5, 1, 0.125), np.arange(1, 2, 0.25), np.arange(2, 4, 0.5),
                       np.arange(4, 8, 1.0), np.arange(8, 16, 2.0), np.arange(16, 32, 4.0)]).astype(np.float32),
}


def f32_to_f6_codes(x: np.ndarray, dtype: int) -> np.ndarray:
    """Nearest code of each fp32 value in OCP E2M3 (dtype 6) or E3M2 (dtype 7): ties to the even code, magnitudes beyond
    the largest saturate, NaN -> +0; uint8 in 0..63 (sign in bit 5), one code per element (not yet packed)."""
    table = _F6_VALUES[dtype]
    x = np.nan_to_num(np.ascontiguousarray(x, dtype=np.float32), nan=0.0)
    a = np.minimum(np.abs(x), table[-1])
    mids = (table[:-1].astype(np.float64) + table[1:].astype(np.float64)) / 2.0
    a64 = a.astype(np.float64)
    code = np.searchsorted(mids, a64, side="left").astype(np.uint8)                       # a == mid -> the lower code
    tie = (mids[np.minimum(code, len(mids) - 1)] == a64) & (code % 2 == 1)                # on a midpoint, lower code odd: the even one above
    code = code + tie.astype(np.uint8)
    return code | (np.signbit(x).astype(np.uint8) << np.uint8(5))


def f6_codes_to_f32(codes: np.ndarray, dtype: int) -> np.ndarray:
    c = np.ascontiguousarray(codes, dtype=np.uint8)
    v = _F6_VALUES[dtype][c & np.uint8(31)]
    return np.where((c >> np.uint8(5)) & np.uint8(1) == 1, -v, v).astype(np.float32)


def pack_f6(codes: np.ndarray) -> np.ndarray:
    """Four 6-bit codes to three bytes along the last axis, as one little-endian bit stream (element i in bits 6 i ..
    6 i + 5); the last axis must be a multiple of 4."""
    c = np.ascontiguousarray(codes, dtype=np.uint8).astype(np.uint32)
    if c.shape[-1] % 4:
        raise ValueError("a multiple of four 6-bit elements per row expected")
    word = c[..., 0::4] | (c[..., 1::4] << 6) | (c[..., 2::4] << 12) | (c[..., 3::4] << 18)       # 24 bits
    out = np.empty(c.shape[:-1] + (c.shape[-1] // 4, 3), dtype=np.uint8)
    for t in range(3):
        out[..., t] = (word >> (8 * t)) & 0xFF
    return out.reshape(c.shape[:-1] + (c.shape[-1] // 4 * 3,))


def unpack_f6(packed: np.ndarray) -> np.ndarray:
    p = np.ascontiguousarray(packed, dtype=np.uint8)
    g = p.reshape(p.shape[:-1] + (p.shape[-1] // 3, 3)).astype(np.uint32)
    word = g[..., 0] | (g[..., 1] << 8) | (g[..., 2] << 16)
    out = np.empty(p.shape[:-1] + (p.shape[-1] // 3, 4), dtype=np.uint8)
    for t in range(4):
        out[..., t] = (word >> (6 * t)) & 63
    return out.reshape(p.shape[:-1] + (p.shape[-1] // 3 * 4,))


def mx_quantize(x: np.ndarray, dtype: int, block: int = 32):
    """Block-scaled storage of an fp32 matrix [rows, K] in the way of the OCP microscaling formats: every `block`
    consecutive elements of a row share an E8M0 scale 2^(floor(log2(max |x|)) - emax) with emax the largest exponent of
    the element type (2 for E2M1 and E2M3, 4 for E3M2, 8 for E4M3, 15 for E5M2), and the elements are x / scale rounded to that type.  Returns (stored
    elements as to_bits would give them, scale codes uint8 [rows, ceil(K / block)]).  An all-zero block gets scale code 127."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    rows, K = x.shape
    nb = (K + block - 1) // block
    pad = np.zeros((rows, nb * block), dtype=np.float32)
    pad[:, :K] = x
    amax = np.abs(pad.reshape(rows, nb, block)).max(axis=2)
    emax = {DTYPE_F4E2M1: 2, DTYPE_F6E2M3: 2, DTYPE_F6E3M2: 4, DTYPE_F8E5M2: 15}.get(dtype, 8)
    with np.errstate(divide="ignore"):
        e = np.where(amax > 0, np.floor(np.log2(np.where(amax > 0, amax, 1.0))) - emax, 0.0)
    e = np.clip(e, -127, 127)
    scale = np.exp2(e).astype(np.float32)
    q = (pad.reshape(rows, nb, block) / scale[:, :, None]).reshape(rows, nb * block)[:, :K]
    if dtype == DTYPE_F8E5M2:
        q = np.clip(q, -57344.0, 57344.0)                # saturating conversion, as the other two encoders do by themselves
    return to_bits(q, dtype), (e + 127).astype(np.uint8)


def to_bits(x, dtype):
    """Storage of an fp32 array in the given dtype: fp32 itself, the uint16 patterns of bf16 / fp16, the uint8
    patterns of E4M3 / E5M2, E2M1 codes packed two to a byte (last axis halved), or 6-bit codes packed four to three bytes."""
    if dtype == DTYPE_F4E2M1:
        return pack_f4(f32_to_f4e2m1_codes(x))
    if dtype in (DTYPE_F6E2M3, DTYPE_F6E3M2):
        return pack_f6(f32_to_f6_codes(x, dtype))
    if dtype == DTYPE_BF16:
        return f32_to_bf16_bits(x)
    if dtype == DTYPE_F16:
        return f32_to_f16_bits(x)
    if dtype == DTYPE_F8E4M3:
        return f32_to_f8e4m3_bits(x)
    if dtype == DTYPE_F8E5M2:
        return f32_to_f8e5m2_bits(x)
    return np.ascontiguousarray(x, dtype=np.float32)


def from_bits(b, dtype):
    """fp32 values of stored data (inverse of to_bits)."""
    if dtype == DTYPE_F4E2M1:
        return f4e2m1_codes_to_f32(unpack_f4(b))
    if dtype in (DTYPE_F6E2M3, DTYPE_F6E3M2):
        return f6_codes_to_f32(unpack_f6(b), dtype)
    if dtype == DTYPE_BF16:
        return bf16_bits_to_f32(b)
    if dtype == DTYPE_F16:
        return f16_bits_to_f32(b)
    if dtype == DTYPE_F8E4M3:
        return f8e4m3_bits_to_f32(b)
    if dtype == DTYPE_F8E5M2:
        return f8e5m2_bits_to_f32(b)
    return np.asarray(b, dtype=np.float32)


def sample_entries(seed, count, batch, M, N, tile_m=256, tile_n=256):
    """(b, i, j) int64 triples to verify when the full output is too large to check:
    `count` iid uniform draws, plus the four corners of every batch's first and last
    matrix and the last row/column entry of every tile row/column, so that no
    workgroup tile goes unchecked."""
    k = _key(seed, "sample", 0)
    ctr = np.arange(3 * count, dtype=np.uint64)
    u = _u01(k, ctr).reshape(3, count)
    b = np.minimum((u[0] * batch).astype(np.int64), batch - 1)
    i = np.minimum((u[1] * M).astype(np.int64), M - 1)
    j = np.minimum((u[2] * N).astype(np.int64), N - 1)
    eb, ei, ej = [], [], []
    for bb in sorted({0, batch - 1}):
        for ii in (0, M - 1):
            for jj in (0, N - 1):
                eb.append(bb); ei.append(ii); ej.append(jj)
        rows = sorted({min(M - 1, t + tile_m - 1) for t in range(0, M, tile_m)})
        cols = sorted({min(N - 1, t + tile_n - 1) for t in range(0, N, tile_n)})
        for ii in rows:
            for jj in cols:
                eb.append(bb); ei.append(ii); ej.append(jj)
    b = np.concatenate([b, np.asarray(eb, dtype=np.int64)])
    i = np.concatenate([i, np.asarray(ei, dtype=np.int64)])
    j = np.concatenate([j, np.asarray(ej, dtype=np.int64)])
    return b, i, j


# ----------------------------------------------------------------------------------------------
# The five workloads

DTYPE_F32, DTYPE_BF16, DTYPE_F16, DTYPE_F8E4M3, DTYPE_F4E2M1, DTYPE_F8E5M2, DTYPE_F6E2M3, DTYPE_F6E3M2 = 0, 1, 2, 3, 4, 5, 6, 7
ACT_NONE, ACT_RELU, ACT_GELU_TANH, ACT_SILU = 0, 1, 2, 3
LAYOUT_RR, LAYOUT_RC, LAYOUT_CR, LAYOUT_CC = 0, 1, 2, 3


@dataclass
class Workload:
    """Host arrays in storage order.  A is stored [M, lda] (row-major) or [K, lda]
    (column-major); B likewise [K, ldb] or [N, ldb]; bias [batch, N] fp32; element
    type fp32, or uint16 holding bf16 bits."""
    name: str
    batch: int
    M: int
    N: int
    K: int
    dtype: int
    act: int
    layout: int
    seed: int
    A: np.ndarray = field(repr=False)
    B: np.ndarray = field(repr=False)
    bias: np.ndarray = field(repr=False)
    check: str = "full"          # "full" or "sampled"

    @property
    def flops(self):
        return 2 * self.batch * self.M * self.N * self.K

    @property
    def algorithmic_bytes(self):
        """One read of A, B and bias, one write of C."""
        es = {DTYPE_F32: 4, DTYPE_F8E4M3: 1, DTYPE_F8E5M2: 1, DTYPE_F4E2M1: 0.5, DTYPE_F6E2M3: 0.75, DTYPE_F6E3M2: 0.75}.get(self.dtype, 2)      # A and B
        cs = 4 if self.dtype == DTYPE_F32 else 2                      # C
        per = int((self.M * self.K + self.K * self.N) * es) + self.M * self.N * cs + 4 * self.N
        return self.batch * per


def _store(x, dtype, transpose=False):
    if transpose:
        x = np.ascontiguousarray(np.swapaxes(x, -1, -2))
    return to_bits(x, dtype)


WORKLOADS = ("c1_f32_256_relu", "c2_f32_skinny16_silu", "c3_f32_4096_rc_gelu",
             "c4_bf16_8192_silu", "c5_bf16_batched32_relu")
BREADTH_WORKLOADS = ("c4_f16_8192_silu", "c2_bf16_skinny16_silu", "c4_f8_8192_rc_silu", "c4_bf8_8192_rc_silu", "c4_bf16_8192_cr_silu",
                     "c2_f32_skinny16_rc_silu", "c4_f4_8192_rc_silu", "c4_f6_8192_rc_silu", "c4_bf6_8192_rc_silu",
                     "c2_f6_skinny16_rc_silu", "c4_bf16_4352_tail_silu")     # further dtypes and shapes


# shape of every workload without its data: (batch, M, N, K, layout, dtype, act)
SPECS = {
    "c1_f32_256_relu": (1, 256, 256, 256, LAYOUT_RR, DTYPE_F32, ACT_RELU),
    "c2_f32_skinny16_silu": (1, 16, 16384, 16384, LAYOUT_RR, DTYPE_F32, ACT_SILU),
    "c3_f32_4096_rc_gelu": (1, 4096, 4096, 4096, LAYOUT_RC, DTYPE_F32, ACT_GELU_TANH),
    "c4_bf16_8192_silu": (1, 8192, 8192, 8192, LAYOUT_RR, DTYPE_BF16, ACT_SILU),
    "c5_bf16_batched32_relu": (32, 2048, 2048, 512, LAYOUT_RR, DTYPE_BF16, ACT_RELU),
    "c4_f16_8192_silu": (1, 8192, 8192, 8192, LAYOUT_RR, DTYPE_F16, ACT_SILU),
    "c2_bf16_skinny16_silu": (1, 16, 16384, 16384, LAYOUT_RR, DTYPE_BF16, ACT_SILU),
    "c4_f8_8192_rc_silu": (1, 8192, 8192, 8192, LAYOUT_RC, DTYPE_F8E4M3, ACT_SILU),
    "c4_bf8_8192_rc_silu": (1, 8192, 8192, 8192, LAYOUT_RC, DTYPE_F8E5M2, ACT_SILU),
    "c4_bf16_8192_cr_silu": (1, 8192, 8192, 8192, LAYOUT_CR, DTYPE_BF16, ACT_SILU),
    "c4_f4_8192_rc_silu": (1, 8192, 8192, 8192, LAYOUT_RC, DTYPE_F4E2M1, ACT_SILU),
    "c4_f6_8192_rc_silu": (1, 8192, 8192, 8192, LAYOUT_RC, DTYPE_F6E2M3, ACT_SILU),
    "c4_bf6_8192_rc_silu": (1, 8192, 8192, 8192, LAYOUT_RC, DTYPE_F6E3M2, ACT_SILU),
    "c2_f6_skinny16_rc_silu": (1, 16, 16384, 16384, LAYOUT_RC, DTYPE_F6E2M3, ACT_SILU),
    "c4_bf16_4352_tail_silu": (1, 4352, 4352, 8192, LAYOUT_RR, DTYPE_BF16, ACT_SILU),
    "c2_f32_skinny16_rc_silu": (1, 16, 16384, 16384, LAYOUT_RC, DTYPE_F32, ACT_SILU),
}


def make_workload(name: str, scale: int = 1) -> Workload:
    """Build one of the five workloads.  `scale` > 1 divides every dimension (for
    quick functional runs at the same distributions); the distributions' parameters that
    depend on K (config 2's variance 1/K) follow the scaled K."""
    s = scale
    if name == "c1_f32_256_relu":
        M = N = K = 256 // s
        return Workload(name, 1, M, N, K, DTYPE_F32, ACT_RELU, LAYOUT_RR, 0,
                        _store(uniform(0, "A", M, K), DTYPE_F32),
                        _store(uniform(0, "B", K, N), DTYPE_F32),
                        uniform(0, "bias", 1, N))
    if name == "c2_f32_skinny16_silu":
        M, N, K = 16, 16384 // s, 16384 // s
        sd = K ** -0.5
        return Workload(name, 1, M, N, K, DTYPE_F32, ACT_SILU, LAYOUT_RR, 1,
                        _store(normal(1, "A", M, K, 0.0, sd), DTYPE_F32),
                        _store(normal(1, "B", K, N, 0.0, sd), DTYPE_F32),
                        uniform(1, "bias", 1, N, -0.1, 0.1))
    if name == "c3_f32_4096_rc_gelu":
        M = N = K = 4096 // s
        return Workload(name, 1, M, N, K, DTYPE_F32, ACT_GELU_TANH, LAYOUT_RC, 2,
                        _store(uniform(2, "A", M, K), DTYPE_F32),
                        _store(uniform(2, "B", K, N), DTYPE_F32, transpose=True),
                        normal(2, "bias", 1, N), check="full" if s >= 4 else "sampled")
    if name == "c4_bf16_8192_silu":
        M = N = K = 8192 // s
        return Workload(name, 1, M, N, K, DTYPE_BF16, ACT_SILU, LAYOUT_RR, 3,
                        _store(normal(3, "A", M, K), DTYPE_BF16),
                        _store(normal(3, "B", K, N), DTYPE_BF16),
                        normal(3, "bias", 1, N), check="full" if s >= 8 else "sampled")
    if name == "c2_f32_skinny16_rc_silu":      # config 2 with B stored column-major ([N][K]: one contiguous K-vector per output)
        M, N, K = 16, 16384 // s, 16384 // s
        sd = K ** -0.5
        return Workload(name, 1, M, N, K, DTYPE_F32, ACT_SILU, LAYOUT_RC, 1,
                        _store(normal(1, "A", M, K, 0.0, sd), DTYPE_F32),
                        _store(normal(1, "B", K, N, 0.0, sd), DTYPE_F32, transpose=True),
                        uniform(1, "bias", 1, N, -0.1, 0.1))
    if name == "c2_bf16_skinny16_silu":        # config 2's shape and distributions in bf16 storage
        M, N, K = 16, 16384 // s, 16384 // s
        sd = K ** -0.5
        return Workload(name, 1, M, N, K, DTYPE_BF16, ACT_SILU, LAYOUT_RR, 1,
                        _store(normal(1, "A", M, K, 0.0, sd), DTYPE_BF16),
                        _store(normal(1, "B", K, N, 0.0, sd), DTYPE_BF16),
                        uniform(1, "bias", 1, N, -0.1, 0.1))
    if name == "c4_f8_8192_rc_silu":           # config 4's shape in 8-bit E4M3 operands (bf16 result), B column-major
        M = N = K = 8192 // s
        return Workload(name, 1, M, N, K, DTYPE_F8E4M3, ACT_SILU, LAYOUT_RC, 3,
                        _store(normal(3, "A", M, K), DTYPE_F8E4M3),
                        _store(normal(3, "B", K, N), DTYPE_F8E4M3, transpose=True),
                        normal(3, "bias", 1, N), check="full" if s >= 8 else "sampled")
    if name == "c4_bf8_8192_rc_silu":          # config 4's shape in 8-bit E5M2 operands (bf16 result), B column-major
        M = N = K = 8192 // s
        return Workload(name, 1, M, N, K, DTYPE_F8E5M2, ACT_SILU, LAYOUT_RC, 3,
                        _store(normal(3, "A", M, K), DTYPE_F8E5M2),
                        _store(normal(3, "B", K, N), DTYPE_F8E5M2, transpose=True),
                        normal(3, "bias", 1, N), check="full" if s >= 8 else "sampled")
    if name == "c4_f4_8192_rc_silu":           # config 4's shape in 4-bit E2M1 operands (bf16 result), k contiguous in both
        M = N = K = 8192 // s
        return Workload(name, 1, M, N, K, DTYPE_F4E2M1, ACT_SILU, LAYOUT_RC, 3,
                        _store(normal(3, "A", M, K), DTYPE_F4E2M1),                  # N(0, 1) rounded to 0, 0.5 .. 6
                        _store(normal(3, "B", K, N), DTYPE_F4E2M1, transpose=True),
                        normal(3, "bias", 1, N), check="full" if s >= 16 else "sampled")
    if name in ("c4_f6_8192_rc_silu", "c4_bf6_8192_rc_silu"):      # config 4's shape in 6-bit E2M3 / E3M2 operands (bf16 result)
        dt = DTYPE_F6E2M3 if name == "c4_f6_8192_rc_silu" else DTYPE_F6E3M2
        M = N = K = 8192 // s
        return Workload(name, 1, M, N, K, dt, ACT_SILU, LAYOUT_RC, 3,
                        _store(normal(3, "A", M, K), dt), _store(normal(3, "B", K, N), dt, transpose=True),
                        normal(3, "bias", 1, N), check="full" if s >= 16 else "sampled")
    if name == "c2_f6_skinny16_rc_silu":       # config 2's shape in 6-bit E2M3 operands, k contiguous in both: bound by reading B once
        M, N, K = 16, 16384 // s, 16384 // s
        return Workload(name, 1, M, N, K, DTYPE_F6E2M3, ACT_SILU, LAYOUT_RC, 3,
                        _store(normal(3, "A", M, K), DTYPE_F6E2M3), _store(normal(3, "B", K, N), DTYPE_F6E2M3, transpose=True),
                        normal(3, "bias", 1, N), check="full" if s >= 8 else "sampled")
    if name == "c4_bf16_4352_tail_silu":       # 17 x 17 tiles of 256 x 256: one more than a round of 256, K as in config 4
        M = N = 4352 // s; K = 8192 // s
        return Workload(name, 1, M, N, K, DTYPE_BF16, ACT_SILU, LAYOUT_RR, 3,
                        _store(normal(3, "A", M, K), DTYPE_BF16), _store(normal(3, "B", K, N), DTYPE_BF16),
                        normal(3, "bias", 1, N), check="full" if s >= 8 else "sampled")
    if name == "c4_bf16_8192_cr_silu":         # config 4 with A stored column-major ([K][M])
        M = N = K = 8192 // s
        return Workload(name, 1, M, N, K, DTYPE_BF16, ACT_SILU, LAYOUT_CR, 3,
                        _store(normal(3, "A", M, K), DTYPE_BF16, transpose=True),
                        _store(normal(3, "B", K, N), DTYPE_BF16),
                        normal(3, "bias", 1, N), check="full" if s >= 8 else "sampled")
    if name == "c4_f16_8192_silu":             # config 4's shape and distributions in binary16 storage
        M = N = K = 8192 // s
        return Workload(name, 1, M, N, K, DTYPE_F16, ACT_SILU, LAYOUT_RR, 3,
                        _store(normal(3, "A", M, K), DTYPE_F16),
                        _store(normal(3, "B", K, N), DTYPE_F16),
                        normal(3, "bias", 1, N), check="full" if s >= 8 else "sampled")
    if name == "c5_bf16_batched32_relu":
        nb, M, N, K = 32, 2048 // s, 2048 // s, 512 // s
        return Workload(name, nb, M, N, K, DTYPE_BF16, ACT_RELU, LAYOUT_RR, 4,
                        _store(uniform(4, "A", M, K, batch=nb), DTYPE_BF16),
                        _store(uniform(4, "B", K, N, batch=nb), DTYPE_BF16),
                        uniform(4, "bias", 1, N, batch=nb).reshape(nb, N),
                        check="full" if s >= 4 else "sampled")
    raise KeyError(name)
