"""The per-device workspace: a graph captured before the library's buffer grows still replays correctly (the old
buffer is retired, not freed); a call that would have to grow the buffer while its stream is being captured is
refused and leaves the capture intact; a caller-supplied buffer is used as it is and never outgrown."""
import numpy as np
import pytest
import torch

from paper_2602_12305_amd import binding as ob
from inputs import synth

pytestmark = pytest.mark.gpu


def skinny(seed, N, K):
    """An fp32 16-row problem whose streaming kernel splits k over the grid: partial sums in the workspace."""
    A = torch.from_numpy(synth.normal(seed, "A", 16, K, 0.0, K ** -0.5)).cuda()
    B = torch.from_numpy(synth.normal(seed, "B", K, N, 0.0, K ** -0.5)).cuda()
    bias = torch.from_numpy(synth.uniform(seed, "bias", 1, N)[0]).cuda()
    C = torch.empty((16, N), dtype=torch.float32, device="cuda")
    return A, B, bias, C


def run_skinny(t, N, K, stream=None):
    A, B, bias, C = t
    ob.optiml_gemm_epilogue(16, N, K, A, K, B, N, bias, C, N, 0, synth.ACT_SILU, stream)


def outgrowing_problem():
    """A bf16 problem with a column-major A whose row-major copy is larger than the workspace in use."""
    have = ob.optiml_workspace_bytes()
    if have > (1 << 30):
        pytest.skip("the workspace already holds more than 1 GiB")
    M, N = 512, 256
    K = ((have // (2 * M)) // 256 + 2) * 256
    A = torch.zeros((K, M), dtype=torch.int16, device="cuda")
    A[:, :] = 0x3F80                                            # bf16 1.0
    B = torch.zeros((K, N), dtype=torch.int16, device="cuda")
    B[::2, :] = 0x3F80
    B[1::2, :] = -0x4080                                        # bf16 -1.0: every sum is exactly 0
    C = torch.full((M, N), 7, dtype=torch.int16, device="cuda")
    xa = ob.variant_names().index("xa_ring")
    args = (1, M, N, K, A, M, 0, B, N, 0, None, 0, C, N, 0, synth.LAYOUT_CR, 1, synth.ACT_NONE, xa)
    assert ob.optiml_variant_supports(xa, *args[:-1]) == ob.OK
    return args, C, 2 * M * K


def test_graph_captured_before_the_workspace_grows_still_replays():
    ob.optiml_set_workspace(None, 0)
    small = skinny(70, 1024, 4096)
    run_skinny(small, 1024, 4096)                               # eager: the workspace exists
    torch.cuda.synchronize()
    want = small[3].clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        run_skinny(small, 1024, 4096)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run_skinny(small, 1024, 4096)
    torch.cuda.synchronize()
    args, C, need = outgrowing_problem()
    before = ob.optiml_workspace_bytes()
    ob.optiml_gemm_epilogue_variant(*args)                      # grows the library's buffer
    torch.cuda.synchronize()
    assert ob.optiml_workspace_bytes() >= max(need, 2 * before) > before
    assert int(C.abs().max().item()) == 0
    filler = torch.full((64 << 20,), 0x7FC00000, dtype=torch.int32, device="cuda")     # would land in a freed buffer
    for rep in range(3):
        small[3].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(small[3], want), rep
    del filler


def test_growth_is_refused_while_the_stream_is_capturing():
    ob.optiml_set_workspace(None, 0)
    small = skinny(71, 1024, 4096)
    run_skinny(small, 1024, 4096)
    torch.cuda.synchronize()
    want = small[3].clone()
    args, C, _ = outgrowing_problem()
    before = ob.optiml_workspace_bytes()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run_skinny(small, 1024, 4096)
            with pytest.raises(ob.OptimlError) as err:
                ob.optiml_gemm_epilogue_variant(*args)
            assert err.value.status == ob.ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert ob.optiml_workspace_bytes() == before
    small[3].zero_()
    graph.replay()                                              # the capture survived the refused call
    torch.cuda.synchronize()
    assert torch.equal(small[3], want)
    assert int(C.min().item()) == 7                             # and the refused call wrote nothing


def test_caller_supplied_workspace_is_used_and_never_outgrown():
    ob.optiml_set_workspace(None, 0)
    t = skinny(72, 2048, 8192)
    run_skinny(t, 2048, 8192)
    torch.cuda.synchronize()
    want = t[3].clone()
    mine = torch.full((4 << 20,), 0x7FC00000, dtype=torch.int32, device="cuda")         # 16 MiB of NaN patterns
    try:
        ob.optiml_set_workspace(mine, mine.numel() * 4)
        assert ob.optiml_workspace_bytes() == mine.numel() * 4
        t[3].zero_()
        run_skinny(t, 2048, 8192)
        torch.cuda.synchronize()
        assert torch.equal(t[3], want)
        assert int((mine != 0x7FC00000).sum().item()) > 0       # the partial sums went through the caller's buffer
        ob.optiml_set_workspace(mine, 4096)                     # too small for the partial sums
        t[3].fill_(5.0)
        with pytest.raises(ob.OptimlError) as err:
            run_skinny(t, 2048, 8192)
        assert err.value.status == ob.ERR_UNSUPPORTED
        torch.cuda.synchronize()
        assert float(t[3].min().item()) == 5.0
    finally:
        ob.optiml_set_workspace(None, 0)
    t[3].zero_()
    run_skinny(t, 2048, 8192)
    torch.cuda.synchronize()
    assert torch.equal(t[3], want)
