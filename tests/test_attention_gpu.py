"""Parity of multi-head self-attention (paper Table 4, task 6) with the CPU oracle, through the C-ABI.

Bars (E1 = max |y - ref| / max(|ref|, rms(ref)), as for the contraction).  bf16 matrix-pipe kernel: the output is
rounded to bf16 (2^-9 relative) and the softmax weights are rounded to bf16 before the second product (each
weight 2^-9 relative, the weighted mean of values inherits at most that times the spread of the values): E1 <=
2e-2.  fp32 kernel: fp32 dot products of d_k terms, hardware exp2 (1 ulp) of a score carrying 1e-7 * |score| of
rounding, fp32 weighted sums: E1 <= 1e-5 for the score ranges tested (|score| < 30).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_12305_amd import binding as ob
from inputs import synth

pytestmark = pytest.mark.gpu
F32, BF16, F16 = 0, 1, 2


def e1(y, ref):
    rho = float(np.sqrt(np.mean(ref * ref))) or 1.0
    return float(np.max(np.abs(y - ref) / np.maximum(np.abs(ref), rho)))


def run(Q, K, V, heads, dtype):
    batch, N, d = Q.shape
    if dtype != F32:
        conv = lambda a: torch.from_numpy(synth.to_bits(a, dtype).view(np.int16)).cuda()
        O = torch.full((batch, N, d), 0x4640, dtype=torch.int16, device="cuda")
    else:
        conv = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
        O = torch.full((batch, N, d), 12345.0, dtype=torch.float32, device="cuda")
    ob.optiml_mhsa(batch, N, d, heads, conv(Q), conv(K), conv(V), O, dtype)
    torch.cuda.synchronize()
    o = O.cpu().numpy()
    return synth.from_bits(o.view(np.uint16), dtype).astype(np.float64) if dtype != F32 else o.astype(np.float64)


def reference(Q, K, V, heads, dtype):
    if dtype != F32:
        return oracle.mhsa(synth.to_bits(Q, dtype), synth.to_bits(K, dtype), synth.to_bits(V, dtype), heads, dtype=dtype)
    return oracle.mhsa(Q, K, V, heads)


def inputs(seed, batch, N, d, qscale=1.0):
    Q = synth.normal(seed, "q", N, d, batch=batch) * np.float32(qscale)
    return Q, synth.normal(seed, "k", N, d, batch=batch), synth.normal(seed, "v", N, d, batch=batch)


@pytest.mark.parametrize("batch,N,d,heads", [(1, 128, 128, 1), (2, 200, 256, 2), (1, 64, 128, 2), (1, 1, 128, 1),
                                             (1, 333, 512, 4), (3, 130, 64, 1), (1, 1000, 256, 4), (1, 65, 384, 3),
                                             (2, 300, 512, 4), (1, 260, 1024, 16), (3, 129, 1024, 8)])
def test_bf16_matrix_pipe_kernel_matches_the_oracle(batch, N, d, heads):
    Q, K, V = inputs(2000 + N + d, batch, N, d)
    got = run(Q, K, V, heads, BF16)
    ref = reference(Q, K, V, heads, BF16)
    assert np.all(np.isfinite(got))
    assert e1(got, ref) <= 2e-2


@pytest.mark.parametrize("dtype", [BF16, F16])
@pytest.mark.parametrize("batch,N,d,heads", [(1, 256, 128, 1), (2, 257, 256, 2), (1, 319, 128, 1), (1, 320, 128, 1), (3, 511, 128, 1),
                                             (1, 513, 384, 3), (1, 1217, 128, 1)])
def test_eight_wave_kernel_at_the_edges_of_its_blocks(batch, N, d, heads, dtype):
    """d_k = 128 and N >= 256 run the kernel whose workgroup holds 256 queries in two groups of waves a phase apart:
    one full block exactly, a last query block of 1 .. 255 rows, a last key block of 1 .. 63 keys, an odd and an even
    number of key blocks."""
    Q, K, V = inputs(2700 + N + d, batch, N, d)
    got = run(Q, K, V, heads, dtype)
    ref = reference(Q, K, V, heads, dtype)
    assert np.all(np.isfinite(got))
    assert e1(got, ref) <= (2e-2 if dtype == BF16 else 2e-3)
    assert np.array_equal(got, run(Q, K, V, heads, dtype))                 # bitwise repeatable


@pytest.mark.parametrize("batch,N,d,heads,dtype", [(1, 100, 96, 3, F32), (2, 77, 40, 5, F32), (1, 300, 128, 1, F32),
                                                   (1, 64, 512, 2, F32), (1, 150, 96, 3, BF16), (1, 5, 7, 1, F32),
                                                   (1, 1, 16, 2, F32), (2, 129, 200, 1, F32)])
def test_fallback_kernel_matches_the_oracle(batch, N, d, heads, dtype):
    Q, K, V = inputs(2100 + N + d, batch, N, d, qscale=0.5)
    got = run(Q, K, V, heads, dtype)
    ref = reference(Q, K, V, heads, dtype)
    assert e1(got, ref) <= (1e-5 if dtype == F32 else 2e-2)


@pytest.mark.parametrize("dtype,d,heads", [(BF16, 256, 2), (F32, 96, 2)])
def test_closed_forms_on_the_gpu(dtype, d, heads):
    N = 192
    _, K, V = inputs(2200, 1, N, d)
    # zero queries: every output row is the mean of the value rows (of the stored, rounded values)
    got = run(np.zeros_like(K), K, V, heads, dtype)
    Vs = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(V)).astype(np.float64) if dtype == BF16 else V.astype(np.float64)
    mean = Vs.mean(axis=1, keepdims=True)
    assert np.max(np.abs(got - mean)) <= (2e-2 if dtype == BF16 else 1e-5) * max(1.0, float(np.max(np.abs(mean))))
    # sharp attention: one-hot keys scaled by 16, query i = key pi(i): output row i = value row pi(i)
    dk = d // heads
    n = min(N, dk)
    Kh = np.zeros((1, n, d), dtype=np.float32)
    for h in range(heads):
        Kh[0, np.arange(n), h * dk + np.arange(n)] = 16.0
    perm = (7 * np.arange(n) + 5) % n
    Vh = synth.integers(2201, "v", n, d, -8, 8)[None]                    # exactly representable in bf16
    got = run(Kh[:, perm], Kh, Vh, heads, dtype)
    assert np.max(np.abs(got - Vh[0][perm])) <= 1e-3                       # other weights are e^(-256/sqrt(dk)) each


def test_large_scores_stay_finite_and_repeat_bitwise():
    Q, K, V = inputs(2300, 1, 256, 128, qscale=30.0)                       # scores of several hundred
    a = run(Q, K, V, 1, BF16); b = run(Q, K, V, 1, BF16)
    assert np.all(np.isfinite(a)) and np.array_equal(a, b)
    ref = reference(Q, K, V, 1, BF16)
    assert e1(a, ref) <= 2e-2
    c = run(Q * np.float32(0.02), K, V, 4, F32); d = run(Q * np.float32(0.02), K, V, 4, F32)
    assert np.array_equal(c, d)


@pytest.mark.parametrize("d,heads,ramp", [(128, 1, (0.05, 8.0)), (128, 1, (8.0, 0.05)), (128, 2, (0.05, 8.0))])
def test_score_range_drifting_along_the_keys(d, heads, ramp):
    """Key magnitudes ramp along the sequence, so the largest score seen so far keeps moving (up in small and large
    steps, or not at all after the first block): the kernel's reference point for the exponents must follow."""
    N = 700
    Q, K, V = inputs(2400 + heads, 2, N, d, qscale=2.0)
    K = K * np.linspace(ramp[0], ramp[1], N, dtype=np.float32)[None, :, None]
    got = run(Q, K, V, heads, BF16)
    ref = reference(Q, K, V, heads, BF16)
    assert np.all(np.isfinite(got))
    assert e1(got, ref) <= 2e-2


def test_benchmark_shape_on_sampled_heads():
    """The shape the benchmark times (batch 4, N 4096, d_model 2048, 16 heads): whole heads of sampled (sequence, head)
    pairs against the oracle, which sees one head as a single-head problem of width d_k."""
    batch, N, d, heads = 4, 4096, 2048, 16
    dk = d // heads
    q, k, v = (synth.f32_to_bf16_bits(synth.normal(9, tag, N, d, batch=batch)) for tag in ("q", "k", "v"))
    dev = [torch.from_numpy(a.view(np.int16)).cuda() for a in (q, k, v)]
    O = torch.full((batch, N, d), 0x4640, dtype=torch.int16, device="cuda")
    ob.optiml_mhsa(batch, N, d, heads, dev[0], dev[1], dev[2], O, BF16)
    torch.cuda.synchronize()
    got = synth.bf16_bits_to_f32(O.cpu().numpy().view(np.uint16)).astype(np.float64)
    assert np.all(np.isfinite(got))
    for b, h in ((0, 0), (1, 7), (3, 15)):
        cols = slice(h * dk, (h + 1) * dk)
        part = lambda a: np.ascontiguousarray(a[b:b + 1, :, cols])
        ref = oracle.mhsa(part(q), part(k), part(v), 1, dtype=oracle.BF16)[0]
        assert e1(got[b, :, cols], ref) <= 2e-2, (b, h)


@pytest.mark.parametrize("batch,N,d,heads", [(2, 200, 256, 2), (1, 333, 512, 4), (3, 130, 64, 1), (1, 1000, 256, 4), (1, 150, 96, 3)])
def test_binary16_storage_matches_the_oracle(batch, N, d, heads):
    """fp16 storage: the same kernels with the f16 matrix instruction; weights and output carry 11 significant bits,
    so the bar is the contraction's for this type (1e-3) plus the weights' rounding: E1 <= 2e-3.  The last case
    (d_k = 32) runs the one-wave-per-query kernel."""
    Q, K, V = inputs(2500 + N + d, batch, N, d)
    got = run(Q, K, V, heads, F16)
    ref = reference(Q, K, V, heads, F16)
    assert np.all(np.isfinite(got))
    assert e1(got, ref) <= 2e-3
