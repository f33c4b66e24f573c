"""The sibling workloads at the sizes and with the inputs `bench.py` times them on (same seeds and recipes), against
the CPU oracle: whole results where the oracle finishes in seconds, otherwise the head, the tail and sampled blocks."""
import math

import numpy as np
import pytest
import torch

import bench
import oracle
from paper_2602_12305_amd import binding as ob
from inputs import synth

pytestmark = pytest.mark.gpu
N28 = bench.STREAM_N


def stream_input(tag):
    return synth.uniform(7, tag, N28 >> 16, 1 << 16, -2.0, 2.0).reshape(-1)


def test_elementwise_and_reductions_on_two_to_the_28_floats():
    hx, hy = stream_input("x"), stream_input("y")
    xd, yd = torch.from_numpy(hx).cuda(), torch.from_numpy(hy).cuda()
    od = torch.empty(N28, dtype=torch.float32, device="cuda")
    spans = [slice(0, 1 << 22), slice(N28 // 2 - 12345, N28 // 2 + (1 << 20)), slice(N28 - (1 << 22), N28)]
    ob.optiml_elementwise(N28, xd, od, 0)
    torch.cuda.synchronize()
    for sp in spans:
        assert np.array_equal(od[sp].cpu().numpy(), oracle.elementwise(hx[sp], 0).astype(np.float32))       # ReLU: bit-exact
    ob.optiml_elementwise(N28, xd, od, 1)
    torch.cuda.synchronize()
    for sp in spans:
        ref = oracle.elementwise(hx[sp], 1)
        assert float(np.max(np.abs(od[sp].cpu().numpy().astype(np.float64) - ref) / ref)) <= 4e-7
    out = torch.empty(1, dtype=torch.float32, device="cuda")
    for op, second in ((0, None), (1, yd), (2, yd)):
        ob.optiml_reduce(N28, xd, second, op, out)
        torch.cuda.synchronize()
        ref = oracle.reduce(hx, hy if second is not None else None, op)
        terms = {0: np.abs(hx.astype(np.float64)).sum(), 1: np.abs(hx.astype(np.float64) * hy).sum(),
                 2: ((hx.astype(np.float64) - hy) ** 2).sum() / N28}[op]
        assert abs(out.item() - float(np.float32(ref))) <= float(np.spacing(np.abs(np.float32(ref)))) + 2.0 ** -40 * terms


def test_transpose_of_16384_squared():
    side = 1 << 14
    hx = stream_input("x").reshape(side, side)
    xd = torch.from_numpy(hx).cuda()
    od = torch.empty((side, side), dtype=torch.float32, device="cuda")
    ob.optiml_transpose(side, side, xd, side, od, side, 4)
    torch.cuda.synchronize()
    for r0, c0 in ((0, 0), (side - 512, 0), (0, side - 512), (side - 512, side - 512), (5000, 9000), (8192 - 256, 8192 - 256)):
        want = oracle.transpose(np.ascontiguousarray(hx[r0:r0 + 512, c0:c0 + 512]))
        assert np.array_equal(od[c0:c0 + 512, r0:r0 + 512].cpu().numpy(), want), (r0, c0)
    assert torch.equal(od, xd.t())                                  # and the whole array against the device's own view


@pytest.mark.parametrize("name", list(bench.ROWS))
def test_row_wise_workloads(name):
    rows, cols = bench.ROWS[name]
    hx = synth.normal(8, "x", rows, cols, 0.5, 2.0)
    xd = torch.from_numpy(hx).cuda()
    if name == "s_ce":
        labels = ((7919 * np.arange(rows)) % cols).astype(np.int32)
        out = torch.empty(1, dtype=torch.float32, device="cuda")
        ob.optiml_cross_entropy(rows, cols, xd, cols, torch.from_numpy(labels).cuda(), out)
        torch.cuda.synchronize()
        ref = oracle.cross_entropy(hx, labels)
        assert abs(out.item() - ref) <= 1e-6 + float(np.spacing(np.float32(ref)))
        return
    od = torch.empty_like(xd)
    ob.optiml_layernorm(rows, cols, xd, od, 1e-5)
    torch.cuda.synchronize()
    pick = sorted({0, 1, rows // 2, rows - 1}) if cols > 8192 else list(range(0, rows, max(1, rows // 64)))[:64] + [rows - 1]
    for r in pick:
        ref = oracle.layernorm(hx[r:r + 1], 1e-5)[0]
        got = od[r].cpu().numpy().astype(np.float64)
        assert float(np.max(np.abs(got - ref))) <= 2.4e-7 + 1e-6 * float(np.max(np.abs(ref))), r


@pytest.mark.parametrize("name", list(bench.LCE))
def test_contraction_fused_with_cross_entropy(name):
    M, N, K, dt = bench.LCE[name]
    A = synth.to_bits(synth.normal(10, "A", M, K, 0.0, K ** -0.5), dt)
    B = synth.to_bits(synth.normal(10, "B", K, N), dt)
    bias = synth.normal(10, "bias", 1, N)[0]
    labels = ((7919 * np.arange(M)) % N).astype(np.int32)
    conv = lambda h: torch.from_numpy(h.view(np.int16) if dt else h).cuda()
    out = torch.empty(1, dtype=torch.float32, device="cuda")
    rows = torch.empty(M, dtype=torch.float32, device="cuda")
    ob.optiml_gemm_cross_entropy_rows(M, N, K, conv(A), K, conv(B), N, torch.from_numpy(bias).cuda(), torch.from_numpy(labels).cuda(),
                                      rows, out, 0, dt)
    torch.cuda.synchronize()
    ref_rows = oracle.gemm_cross_entropy_rows(A, B, bias, labels, M, N, K, dtype=dt)
    ref = float(np.mean(ref_rows))
    # unit-variance logits: |bias| + sum |a b| stays below 60, so the bound of tests/test_linear_ce_gpu.py is below 1.2e-4,
    # for the mean and for every single row
    assert math.isfinite(out.item()) and abs(out.item() - ref) <= 1.2e-4, (out.item(), ref)
    err = np.abs(rows.cpu().numpy().astype(np.float64) - ref_rows)
    assert float(err.max()) <= 1.2e-4, (int(err.argmax()), float(err.max()))
    print(f"{name}: worst row {float(err.max()):.3e}, mean {abs(out.item() - ref):.3e}")


@pytest.mark.parametrize("name", list(bench.GLN))
def test_contraction_fused_with_layernorm(name):
    """Whole rows, sampled over the row tiles (first, last and every 37th row): the oracle normalises a row only when it
    has all of it.  Unit-variance products on a bias of spread 3: |bias| + sum |a b| stays below 80, s is about 3.2, so
    the bound of tests/test_linear_ln_gpu.py stays below 2e-4 (1 + |y|); one rounding to the storage type on top."""
    M, N, K, dt = bench.GLN[name]
    A = synth.to_bits(synth.normal(13, "A", M, K, 0.0, K ** -0.5), dt)
    B = synth.to_bits(synth.normal(13, "B", K, N), dt)
    bias = synth.normal(13, "bias", 1, N, 1.5, 3.0)[0]
    conv = lambda h: torch.from_numpy(h.view(np.int16) if dt else h).cuda()
    Y = torch.empty((M, N), dtype=torch.int16 if dt else torch.float32, device="cuda")
    ob.optiml_gemm_layernorm(M, N, K, conv(A), K, conv(B), N, torch.from_numpy(bias).cuda(), Y, N, 1e-5, 0, dt)
    torch.cuda.synchronize()
    rows = sorted(set(range(0, M, 37)) | {M - 1, 255, 256})
    ref = oracle.gemm_layernorm(np.ascontiguousarray(A[rows]), B, bias, len(rows), N, K, dtype=dt, eps=1e-5)
    got = Y[rows].cpu().numpy()
    got = (synth.from_bits(got.view(np.uint16), dt) if dt else got).astype(np.float64)
    half = 2.0 ** -8 if dt else 2.0 ** -24
    err = np.abs(got - ref) - half * np.abs(ref)
    assert np.all(np.isfinite(got)) and float(np.max(err - 2e-4 * (1 + np.abs(ref)))) <= 0.0, float(err.max())
    print(f"{name}: worst entry beyond its rounding step {float(err.max()):.3e} over {len(rows)} rows")
