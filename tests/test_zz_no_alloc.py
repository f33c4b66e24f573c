"""optiml_gemm_epilogue_noalloc (the entry point for callers that cannot allocate device memory) against
optiml_gemm_epilogue_strided_batched: same kernels, scratch in the library's static device array instead of the
workspace, so C must agree bit for bit - on two calls in a row, the second with a smaller input - and a problem
whose scratch does not fit the array is refused without touching C."""
import numpy as np
import pytest
import torch

from paper_2602_12305_amd import binding as ob
from inputs import synth

pytestmark = pytest.mark.gpu

FAKE = 0x10000      # stands for an aligned C where only the dispatcher's choice is asked for


def skinny_problem(seed, batch, M, N, K):
    """fp32, few rows: the streaming kernel splits k over the grid and keeps partial sums in scratch memory."""
    A = torch.from_numpy(synth.normal(seed, "A", M, K, 0.0, K ** -0.5, batch=batch)).cuda()
    B = torch.from_numpy(synth.normal(seed, "B", K, N, 0.0, K ** -0.5, batch=batch)).cuda()
    bias = torch.from_numpy(synth.uniform(seed, "bias", batch, N)).cuda()
    return (batch, M, N, K, A, K, M * K, B, N, K * N, bias, N), (batch, M, N)


def both(args, shape, layout, dtype, act, out_dtype):
    ref = torch.zeros(shape, dtype=out_dtype, device="cuda")
    got = torch.zeros(shape, dtype=out_dtype, device="cuda")
    _, M, N = shape
    ob.optiml_gemm_epilogue_strided_batched(*args, ref, N, M * N, layout, dtype, act)
    ob.optiml_gemm_epilogue_noalloc(*args, got, N, M * N, layout, dtype, act)
    torch.cuda.synchronize()
    return ref, got


def test_noalloc_matches_the_allocating_entry_point_on_two_calls_in_a_row():
    for seed, batch, M, N, K in ((80, 1, 16, 4096, 8192), (81, 2, 12, 1024, 4096)):      # the second one smaller
        args, shape = skinny_problem(seed, batch, M, N, K)
        name = ob.optiml_variant_name(ob.optiml_select_variant(*args, FAKE, N, M * N, 0, 0, synth.ACT_SILU))
        assert name.startswith("skinny_f32"), name                   # too few column blocks for the chip: k is split over the grid
        ref, got = both(args, shape, 0, 0, synth.ACT_SILU, torch.float32)
        assert float(ref.abs().max().item()) > 0.0
        assert torch.equal(got, ref), (seed, float((got - ref).abs().max().item()))
    # a column-major A with few rows: copy of A plus split-k partial sums behind it, both in the array (bf16)
    M, N, K = 64, 512, 4096                                     # 0.5 MiB copy + at most 8 MiB of partial sums
    At = torch.from_numpy(synth.f32_to_bf16_bits(np.ascontiguousarray(synth.normal(82, "A", M, K, 0.0, K ** -0.5).T)).view(np.int16)).cuda()
    Bm = torch.from_numpy(synth.f32_to_bf16_bits(synth.normal(82, "B", K, N)).view(np.int16)).cuda()
    args = (1, M, N, K, At, M, 0, Bm, N, 0, None, 0)
    assert ob.optiml_variant_name(ob.optiml_select_variant(*args, FAKE, N, 0, synth.LAYOUT_CR, 1, synth.ACT_RELU)) == "xa_ring"
    ref, got = both(args, (1, M, N), synth.LAYOUT_CR, 1, synth.ACT_RELU, torch.int16)
    assert int(ref.abs().max().item()) > 0
    assert torch.equal(got, ref)


def test_noalloc_refuses_what_does_not_fit_its_array():
    M, N, K = 4096, 512, 4096                                   # bf16, A column-major: a 32 MiB copy of A
    At = torch.zeros((K, M), dtype=torch.int16, device="cuda")
    Bm = torch.zeros((K, N), dtype=torch.int16, device="cuda")
    C = torch.full((M, N), 7, dtype=torch.int16, device="cuda")
    args = (1, M, N, K, At, M, 0, Bm, N, 0, None, 0, C, N, 0, synth.LAYOUT_CR, 1, synth.ACT_NONE)
    if ob.optiml_variant_name(ob.optiml_select_variant(*args)) != "xa_ring":
        pytest.skip("the dispatcher no longer copies A for this shape")
    with pytest.raises(ob.OptimlError) as err:
        ob.optiml_gemm_epilogue_noalloc(*args)
    assert err.value.status == ob.ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert int(C.min().item()) == 7 and int(C.max().item()) == 7
    ob.optiml_gemm_epilogue_strided_batched(*args)              # the allocating entry point takes it
    torch.cuda.synchronize()
    assert int(C.abs().max().item()) == 0
