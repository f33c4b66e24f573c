"""The five benchmark workloads at full size, in the launch configuration bench.py times
(the dispatcher's choice), against the CPU oracle: every entry where the oracle finishes in
seconds, otherwise 65,536 seeded sampled entries plus tile corners.  Each shape is also run
on integer-valued inputs, where any fp32 summation order must reproduce the exact result."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_12305_amd import binding as ob
from inputs import synth
from gpu_harness import TOL, c_values, alloc_c, ld_elements, to_dev
from helpers import e1

pytestmark = pytest.mark.gpu


def run_workload(w):
    lda, ldb = ld_elements(w.A, w.dtype), ld_elements(w.B, w.dtype)
    sA = w.A.shape[-2] * lda if w.batch > 1 else 0
    sB = w.B.shape[-2] * ldb if w.batch > 1 else 0
    Ad, Bd, bd = to_dev(w.A), to_dev(w.B), to_dev(w.bias)
    Cd = alloc_c(w.batch, w.M, w.N, w.dtype)
    ob.optiml_gemm_epilogue_strided_batched(w.batch, w.M, w.N, w.K, Ad, lda, sA, Bd, ldb, sB, bd, w.N if w.batch > 1 else 0,
                                            Cd, w.N, w.M * w.N, w.layout, w.dtype, w.act)
    torch.cuda.synchronize()
    first = Cd.clone()
    ob.optiml_gemm_epilogue_strided_batched(w.batch, w.M, w.N, w.K, Ad, lda, sA, Bd, ldb, sB, bd, w.N if w.batch > 1 else 0,
                                            Cd, w.N, w.M * w.N, w.layout, w.dtype, w.act)
    torch.cuda.synchronize()
    assert torch.equal(first, Cd), "two runs of the same call differ bitwise"
    del Ad, Bd
    return c_values(Cd, w.dtype, w.N)[0]


def reference(w, Y):
    """(gpu values, oracle values, oracle's |bias| + sum|a b|) over the checked entries."""
    if w.check == "full":
        ref, den = oracle.gemm_epilogue(w.A, w.B, w.bias, w.M, w.N, w.K, dtype=w.dtype, act=w.act, layout=w.layout,
                                        batch=w.batch, want_absden=True)
        return Y, ref, den
    sb, si, sj = synth.sample_entries(w.seed, 65536, w.batch, w.M, w.N)
    ref, den = oracle.gemm_epilogue_sampled(sb, si, sj, w.A, w.B, w.bias, w.M, w.N, w.K, dtype=w.dtype, act=w.act,
                                            layout=w.layout, batch=w.batch, want_absden=True)
    return Y[sb, si, sj], ref, den


FULL_CHECK = {"c1_f32_256_relu": "full", "c2_f32_skinny16_silu": "full", "c3_f32_4096_rc_gelu": "full",
              "c4_bf16_8192_silu": "sampled", "c5_bf16_batched32_relu": "full", "c4_f16_8192_silu": "sampled", "c2_bf16_skinny16_silu": "full", "c4_f8_8192_rc_silu": "sampled", "c4_bf8_8192_rc_silu": "sampled", "c4_f6_8192_rc_silu": "sampled", "c4_bf6_8192_rc_silu": "sampled", "c2_f6_skinny16_rc_silu": "sampled", "c4_bf16_8192_cr_silu": "sampled", "c2_f32_skinny16_rc_silu": "full", "c4_f4_8192_rc_silu": "sampled", "c4_bf16_4352_tail_silu": "sampled"}


@pytest.mark.parametrize("name", synth.WORKLOADS + synth.BREADTH_WORKLOADS)
def test_workload_matches_oracle(name):
    w = synth.make_workload(name)
    w.check = FULL_CHECK[name]
    Y = run_workload(w)
    got, ref, den = reference(w, Y)
    assert np.all(np.isfinite(Y))
    err = e1(got, ref)
    # componentwise forward error against |bias| + sum|a b| (fp32 accumulation), plus half a
    # step of the value for the one rounding of a bf16 / binary16 output; below 1e-36 (SiLU of
    # z < -88, where exp(-z) overflows fp32) the kernel may return -0
    half_step = {synth.DTYPE_F32: 0.0, synth.DTYPE_BF16: 2.0 ** -8, synth.DTYPE_F16: 2.0 ** -11,
                 synth.DTYPE_F8E4M3: 2.0 ** -8, synth.DTYPE_F4E2M1: 2.0 ** -8, synth.DTYPE_F8E5M2: 2.0 ** -8,
                 synth.DTYPE_F6E2M3: 2.0 ** -8, synth.DTYPE_F6E3M2: 2.0 ** -8}[w.dtype]     # 8- and 4-bit operands: bf16 result
    step = half_step * 1.01 * np.abs(ref)
    e2 = float(np.max((np.abs(got - ref) - step - 1e-36) / den))
    print(f"{name}: E1 = {err:.3e}, E2 = {e2:.3e} over {ref.size} entries ({w.check})")
    assert err <= TOL[w.dtype]
    assert e2 <= 16 * 2.0 ** -24


@pytest.mark.parametrize("name", synth.WORKLOADS + synth.BREADTH_WORKLOADS)
def test_workload_shape_is_exact_on_integers(name):
    # (the few-row 6-bit shape at half its N and K: its 268 M elements take most of a minute to encode; the full size is
    # checked by test_workload_matches_oracle)
    w = synth.make_workload(name, scale=2 if name == "c2_f6_skinny16_rc_silu" else 1)
    lead = (w.batch,) if w.batch > 1 else ()
    def ints(tag, rows, cols, transpose):
        x = synth.integers(w.seed + 77, tag, rows, cols, batch=w.batch if w.batch > 1 else None)
        if transpose:
            x = np.ascontiguousarray(np.swapaxes(x, -1, -2))
        return synth.to_bits(x, w.dtype)
    w.A = ints("A", w.M, w.K, bool(w.layout & 2))
    w.B = ints("B", w.K, w.N, bool(w.layout & 1))
    w.bias = synth.integers(w.seed + 77, "bias", 1, w.N, -5, 5, batch=w.batch).reshape(w.batch, w.N)
    w.act = synth.ACT_RELU
    w.check = "sampled"
    Y = run_workload(w)
    got, ref, _ = reference(w, Y)
    if w.dtype in (synth.DTYPE_BF16, synth.DTYPE_F8E4M3, synth.DTYPE_F4E2M1, synth.DTYPE_F8E5M2, synth.DTYPE_F6E2M3, synth.DTYPE_F6E3M2):
        ref = synth.bf16_bits_to_f32(oracle.bf16_from_double(ref)).astype(np.float64)
    elif w.dtype == synth.DTYPE_F16:
        ref = oracle.f16_to_double(oracle.f16_from_double(ref))
    assert np.array_equal(got, ref)


def test_dispatcher_choice_is_near_the_fastest_variant_on_a_few_clear_cases():
    """Shapes on which the right family wins by 3x or more (streaming against tiles for a few rows, tiles against
    streaming for thousands): the dispatcher's choice must be within 2.5x of the fastest variant that takes the
    shape.  A coarse guard against a mis-calibrated estimate; the full comparison is `dispatch_check`."""
    from paper_2602_12305_amd import dispatch_check
    for case in dispatch_check.SETS["quick"]:
        pn, pt, bn, bt = dispatch_check.check(*case, steps=10)
        assert pt <= 2.5 * bt, (case, pn, pt, bn, bt)
