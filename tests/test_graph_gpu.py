"""The entry points only enqueue kernels on the caller's stream, so a sequence of calls can be captured into a HIP
graph once the per-device workspace has its size (the first, eager call allocates it; allocation is not allowed under
capture).  Each replay is checked against the eager results, with eager work and synchronisations between replays."""
import numpy as np
import pytest
import torch

from paper_2602_12305_amd import binding as ob
from inputs import synth

pytestmark = pytest.mark.gpu


def test_captured_sequence_of_calls_replays_bit_for_bit():
    M, N, K = 16, 1024, 4096                                    # streaming kernel with a grid split: uses the workspace
    A = torch.from_numpy(synth.normal(50, "A", M, K, 0.0, K ** -0.5)).cuda()
    B = torch.from_numpy(synth.normal(50, "B", K, N, 0.0, K ** -0.5)).cuda()
    bias = torch.from_numpy(synth.uniform(50, "bias", 1, N)[0]).cuda()
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")
    Mb, Nb, Kb = 512, 768, 256                                  # bf16 ring kernel
    Ab = torch.from_numpy(synth.f32_to_bf16_bits(synth.normal(51, "A", Mb, Kb)).view(np.int16)).cuda()
    Bb = torch.from_numpy(synth.f32_to_bf16_bits(synth.normal(51, "B", Kb, Nb)).view(np.int16)).cuda()
    Cb = torch.empty((Mb, Nb), dtype=torch.int16, device="cuda")
    n = (1 << 20) + 7
    x = torch.from_numpy(synth.uniform(52, "x", 1, n)[0]).cuda()
    total = torch.empty(1, dtype=torch.float32, device="cuda")
    labels = torch.from_numpy(((7 * np.arange(Mb)) % Nb).astype(np.int32)).cuda()
    loss = torch.empty(1, dtype=torch.float32, device="cuda")

    def sequence():
        ob.optiml_gemm_epilogue(M, N, K, A, K, B, N, bias, C, N, 0, synth.ACT_SILU)
        ob.optiml_gemm_epilogue(Mb, Nb, Kb, Ab, Kb, Bb, Nb, None, Cb, Nb, 1, synth.ACT_RELU)
        ob.optiml_reduce(n, x, None, 0, total)
        ob.optiml_gemm_cross_entropy(Mb, Nb, Kb, Ab, Kb, Bb, Nb, None, labels, loss, 0, 1)

    sequence()                                                  # eager: sizes the workspace, gives the expected bits
    torch.cuda.synchronize()
    want = [t.clone() for t in (C, Cb, total, loss)]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        sequence()                                              # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            sequence()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in (C, Cb, total, loss):
            t.zero_()                                           # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((C, Cb, total, loss), want):
            assert torch.equal(got, ref), rep


def test_copy_paths_replay_bit_for_bit_under_a_graph():
    """The paths that run several kernels around a copy in the workspace - an odd-sized problem (padded copies, a fast
    kernel, a copy back), a column-major A with few rows (copy, then a streaming kernel whose partial sums sit behind
    the copy) - captured after an eager call has sized the workspace, replayed three times against the eager bits."""
    M, N, K = 131, 517, 1029                                    # bf16, nothing aligned: the padded-copy path
    Ao = torch.from_numpy(synth.f32_to_bf16_bits(synth.normal(60, "A", M, K)).view(np.int16)).cuda()
    Bo = torch.from_numpy(synth.f32_to_bf16_bits(synth.normal(60, "B", K, N)).view(np.int16)).cuda()
    bo = torch.from_numpy(synth.uniform(60, "bias", 1, N)[0]).cuda()
    Co = torch.empty((M, N), dtype=torch.int16, device="cuda")
    Mc, Nc, Kc = 40, 1024, 4096                                 # fp32, A column-major [K][M]: copy, then streamed
    Ac = torch.from_numpy(np.ascontiguousarray(synth.normal(61, "A", Mc, Kc, 0.0, Kc ** -0.5).T)).cuda()
    Bc = torch.from_numpy(synth.normal(61, "B", Kc, Nc, 0.0, Kc ** -0.5)).cuda()
    Cc = torch.empty((Mc, Nc), dtype=torch.float32, device="cuda")
    assert ob.optiml_variant_name(ob.optiml_select_variant(1, M, N, K, Ao, K, 0, Bo, N, 0, bo, 0, Co, N, 0, 0, 1, 3)) == "xpad"
    assert ob.optiml_variant_name(ob.optiml_select_variant(1, Mc, Nc, Kc, Ac, Mc, 0, Bc, Nc, 0, None, 0, Cc, Nc, 0, 2, 0, 1)) == "xa_ring"

    def sequence():
        ob.optiml_gemm_epilogue_ex(M, N, K, Ao, K, Bo, N, bo, Co, N, 0, 1, synth.ACT_SILU)
        ob.optiml_gemm_epilogue_ex(Mc, Nc, Kc, Ac, Mc, Bc, Nc, None, Cc, Nc, 2, 0, synth.ACT_RELU)

    sequence()
    torch.cuda.synchronize()
    want = [t.clone() for t in (Co, Cc)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        sequence()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            sequence()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in (Co, Cc):
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((Co, Cc), want):
            assert torch.equal(got, ref), rep
