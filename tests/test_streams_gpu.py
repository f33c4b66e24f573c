"""Parity of the streaming siblings (element-wise ReLU / sigmoid, sum, dot, MSE; paper Table 4 tasks
10, 1, 14, 15, 7) with the CPU oracle, through the C-ABI.

Bars.  ReLU: bit-exact.  Sigmoid: |y - ref| <= 4e-7 * ref + 1e-45 (fp32 arithmetic around the hardware
exponential and reciprocal: about 3 ulp; results below the smallest normal may flush).  Reductions: the
kernels add fp64 terms in a fixed order and round once, so the result must be within one float step of
the oracle's value rounded to float plus 2^-40 of sum|term| for the fp64 reordering; exact on
integer-valued inputs; bitwise repeatable.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_12305_amd import binding as ob
from inputs import synth

pytestmark = pytest.mark.gpu

SIZES = [1, 2, 3, 4, 5, 63, 64, 1023, 4096, 4099, 65536 + 7, (1 << 20) + 1, 3 * (1 << 20) + 2]


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_ew(x, op, offset=0, inplace=False):
    """offset (elements) shifts both arrays off 16-byte alignment."""
    n = x.size
    xd = torch.zeros(n + offset + 8, dtype=torch.float32, device="cuda")
    xd[offset:offset + n] = dev(x)
    yd = xd if inplace else torch.full((n + offset + 8,), 7.0, dtype=torch.float32, device="cuda")
    ob.optiml_elementwise(n, xd[offset:], yd[offset:], op)
    torch.cuda.synchronize()
    out = yd.cpu().numpy()
    if not inplace:
        assert np.all(out[:offset] == 7.0) and np.all(out[offset + n:] == 7.0)      # nothing written outside
    return out[offset:offset + n]


def run_red(x, y, op, offset=0):
    n = x.size
    xd = torch.zeros(n + offset + 8, dtype=torch.float32, device="cuda"); xd[offset:offset + n] = dev(x)
    yd = None
    if y is not None:
        yd = torch.zeros(n + offset + 8, dtype=torch.float32, device="cuda"); yd[offset:offset + n] = dev(y)
    out = torch.full((3,), 7.0, dtype=torch.float32, device="cuda")
    ob.optiml_reduce(n, xd[offset:], None if yd is None else yd[offset:], op, out[1:])
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert o[0] == 7.0 and o[2] == 7.0
    return np.float32(o[1])


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("offset", [0, 1])
def test_relu_is_bit_exact(n, offset):
    x = synth.normal(900 + n, "x", 1, n)[0]
    x[:: 7] = 0.0
    got = run_ew(x, ob_op("relu"), offset)
    ref = oracle.elementwise(x, oracle.EW_RELU)
    assert np.array_equal(got.astype(np.float64), ref)


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("offset", [0, 3])
def test_sigmoid_matches_the_oracle(n, offset):
    x = synth.uniform(910 + n, "x", 1, n)[0] * np.float32(20.0)
    got = run_ew(x, ob_op("sigmoid"), offset).astype(np.float64)
    ref = oracle.elementwise(x, oracle.EW_SIGMOID)
    assert np.all(np.abs(got - ref) <= 4e-7 * ref + 1e-45)


def test_sigmoid_special_values_and_in_place():
    x = np.array([0.0, -0.0, 88.0, -87.0, -90.0, -104.0, 1e30, -1e30, np.inf, -np.inf, 1e-30], dtype=np.float32)
    got = run_ew(x, ob_op("sigmoid"), 0, inplace=True).astype(np.float64)
    ref = oracle.elementwise(x, oracle.EW_SIGMOID)
    assert got[0] == 0.5 and got[1] == 0.5 and got[2] == 1.0 and got[6] == 1.0 and got[8] == 1.0
    assert got[7] == 0.0 and got[9] == 0.0
    assert np.all(np.isfinite(got))
    big = np.abs(ref) >= 1.2e-38                     # below the smallest normal the result may flush to zero
    assert np.all(np.abs(got[big] - ref[big]) <= 4e-7 * ref[big])
    assert np.all(got[~big] <= 1.2e-38)
    y = synth.normal(920, "x", 1, 5000)[0]
    assert np.array_equal(run_ew(y, ob_op("relu"), 0, inplace=True), np.maximum(y, 0))


def ob_op(name):
    return {"relu": 0, "sigmoid": 1, "sum": 0, "dot": 1, "mse": 2}[name]


def check_reduction(x, y, op, offset=0):
    oop = {0: oracle.RED_SUM, 1: oracle.RED_DOT, 2: oracle.RED_MSE}[op]
    got = run_red(x, y, op, offset)
    ref = oracle.reduce(x, y, oop)
    x64 = x.astype(np.float64)
    if op == 0:
        mass = float(np.sum(np.abs(x64)))
    elif op == 1:
        mass = float(np.sum(np.abs(x64 * y.astype(np.float64))))
    else:
        mass = ref
    ref32 = np.float32(ref)
    step = float(np.spacing(np.abs(ref32))) if np.isfinite(ref32) else 0.0
    assert abs(float(got) - float(ref32)) <= step + mass * 2.0 ** -40, (float(got), ref)
    assert run_red(x, y, op, offset) == got                                          # bitwise repeatable
    return got


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("op", [0, 1, 2])
def test_reductions_match_the_oracle(n, op):
    x = synth.normal(930 + n, "x", 1, n)[0]; y = synth.normal(930 + n, "y", 1, n)[0]
    check_reduction(x, None if op == 0 else y, op, offset=0)
    check_reduction(x, None if op == 0 else y, op, offset=1)                          # unaligned: scalar path


@pytest.mark.parametrize("n", [1, 1000, 65537, (1 << 20) + 3])
def test_reductions_are_exact_on_integers(n):
    x = synth.integers(940 + n, "x", 1, n)[0]; y = synth.integers(940 + n, "y", 1, n)[0]
    assert float(run_red(x, None, 0)) == float(np.sum(x.astype(np.float64)))
    assert float(run_red(x, y, 1)) == float(np.sum(x.astype(np.float64) * y.astype(np.float64)))
    d = x.astype(np.float64) - y.astype(np.float64)
    assert float(run_red(x, y, 2)) == float(np.float32(np.sum(d * d) / n))


def test_reduction_closed_forms_and_cancellation():
    n = 1 << 21
    ones = np.ones(n, dtype=np.float32)
    assert float(run_red(ones, None, 0)) == float(n)
    alt = np.where(np.arange(n + 1) % 2 == 0, 1.0, -1.0).astype(np.float32)
    assert float(run_red(alt, None, 0)) == 1.0                                        # a lost element would show
    big = (synth.normal(950, "x", 1, n)[0].astype(np.float64) * 1e6).astype(np.float32)
    big[::2] = -big[1::2]
    assert float(run_red(big, None, 0)) == 0.0                                        # exact despite 1e6-sized terms
    i = np.arange(5000, dtype=np.float32)
    assert float(run_red(i, i, 1)) == float(np.float32(4999 * 5000 * 9999 / 6))
    assert float(run_red(i, i, 2)) == 0.0


def test_empty_reduction_writes_zero_and_empty_elementwise_writes_nothing():
    out = torch.full((1,), 7.0, dtype=torch.float32, device="cuda")
    for op in (0, 1, 2):
        out.fill_(7.0)
        ob.optiml_reduce(0, None, None, op, out)
        torch.cuda.synchronize()
        assert out.item() == 0.0
    y = torch.full((4,), 7.0, dtype=torch.float32, device="cuda")
    ob.optiml_elementwise(0, y, y, 1)
    torch.cuda.synchronize()
    assert torch.all(y == 7.0)


def test_runs_on_a_side_stream():
    n = 100003
    x = synth.normal(960, "x", 1, n)[0]
    xd = dev(x); out = torch.zeros(1, dtype=torch.float32, device="cuda")
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        ob.optiml_reduce(n, xd, None, 0, out, stream=s)
    s.synchronize()
    ref = np.float32(oracle.reduce(x, None, oracle.RED_SUM))
    assert abs(out.item() - float(ref)) <= float(np.spacing(np.abs(ref)))


@pytest.mark.parametrize("dtype", [np.float32, np.uint16])
@pytest.mark.parametrize("rows,cols,pad_src,pad_dst", [(1, 1, 0, 0), (64, 64, 0, 0), (200, 136, 0, 0), (77, 131, 0, 0), (1000, 8, 8, 16),
                                                      (5, 3000, 3, 1), (1, 4096, 0, 0), (4096, 1, 0, 0), (520, 1032, 8, 8),
                                                      (2104, 4208, 0, 8), (4104, 16400, 0, 8)])
def test_transpose_is_bit_exact(dtype, rows, cols, pad_src, pad_dst):
    """Table 4 task 8: every element at its mirror position, bit for bit (16-bit patterns include NaNs), padding untouched;
    aligned shapes take the vectorised kernel, the others the element-wise one; the last shape is large enough for the
    launch with two tiles per workgroup, with an odd number of column tiles and ragged edges."""
    rng = np.random.default_rng(rows * 7 + cols)
    if dtype == np.float32:
        x = rng.standard_normal((rows, cols + pad_src)).astype(np.float32)
        src = torch.from_numpy(x).cuda(); dst = torch.full((cols, rows + pad_dst), 777.0, dtype=torch.float32, device="cuda")
    else:
        x = rng.integers(0, 1 << 16, size=(rows, cols + pad_src), dtype=np.uint16)
        src = torch.from_numpy(x.view(np.int16)).cuda(); dst = torch.full((cols, rows + pad_dst), 777, dtype=torch.int16, device="cuda")
    ob.optiml_transpose(rows, cols, src, cols + pad_src, dst, rows + pad_dst, x.dtype.itemsize)
    torch.cuda.synchronize()
    got = dst.cpu().numpy().view(x.dtype)
    want = oracle.transpose(np.ascontiguousarray(x[:, :cols]))
    assert np.array_equal(got[:, :rows].view(np.uint8), want.view(np.uint8))
    pad = got[:, rows:]
    assert np.all(pad == (np.float32(777.0) if dtype == np.float32 else np.uint16(777)))
