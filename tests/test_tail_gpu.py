"""The variant that splits the partly filled last round of a tiled contraction along k (`xtail_split`): a main
block by the ordinary tile kernel, the remaining strips as k-split partial products summed in a fixed order.
Checked against the oracle on sampled entries that cover the main block, both strips, their corner and the ragged
edges; exactly on integer-valued inputs (any fp32 summation order must give the same bits), and bitwise repeatable."""
import numpy as np
import pytest
import torch

import oracle
from inputs import synth
from paper_2602_12305_amd import binding as ob
from gpu_harness import TOL, run_gpu
from helpers import e1, store

pytestmark = pytest.mark.gpu
BF16, F16 = synth.DTYPE_BF16, synth.DTYPE_F16


def tail_id():
    return ob.variant_names().index("xtail_split")


def entries(M, N, seed):
    """Sampled (row, column) pairs: a seeded spread plus the borders of the 256-tiles around the main block."""
    _, si, sj = synth.sample_entries(seed, 3000, 1, M, N)
    edge_r = [r for r in (0, 255, 256, M - 258, M - 257, M - 256, M - 255, M - 2, M - 1) if 0 <= r < M]
    edge_c = [c for c in (0, 255, 256, N - 258, N - 257, N - 256, N - 255, N - 2, N - 1) if 0 <= c < N]
    er, ec = np.meshgrid(edge_r, edge_c, indexing="ij")
    i = np.concatenate([si, er.ravel()]); j = np.concatenate([sj, ec.ravel()])
    return np.zeros_like(i), i, j


@pytest.mark.parametrize("dtype,layout,M,N,K", [(BF16, 0, 4352, 4352, 2048), (BF16, 1, 4352, 4352, 2112), (F16, 0, 4104, 4104, 2048),
                                                (BF16, 0, 4352, 4096, 4096), (BF16, 0, 4100, 4360, 4104), (BF16, 5, 4352, 4352, 2048)])
def test_tail_split_matches_the_oracle_on_sampled_entries(dtype, layout, M, N, K):
    vid = tail_id()
    A = synth.normal(6000 + M + K, "A", M, K) * np.float32(K ** -0.5); B = synth.normal(6000 + M + K, "B", K, N)
    bias = synth.normal(6000 + M + K, "bias", 1, N)[0]
    As, Bs = store(A, dtype, False), store(B, dtype, bool(layout & 1))
    P = 0x10000
    ldc = M if layout & 4 else N
    assert ob.lib().optiml_variant_supports(vid, 1, M, N, K, P, As.shape[-1], 0, P, Bs.shape[-1], 0, P, 0, P, ldc, 0, layout, dtype, 3) == 0
    Y1, _, C1 = run_gpu(As, Bs, bias, 1, M, N, K, dtype, synth.ACT_SILU, layout, variant=vid)
    Y2, _, C2 = run_gpu(As, Bs, bias, 1, M, N, K, dtype, synth.ACT_SILU, layout, variant=vid)
    assert torch.equal(C1, C2)                                                  # bitwise repeatable
    sb, si, sj = entries(M, N, 61)
    ref = oracle.gemm_epilogue_sampled(sb, si, sj, As, Bs, bias, M, N, K, dtype=dtype, act=synth.ACT_SILU, layout=layout & 3)
    assert np.all(np.isfinite(Y1))
    assert e1(Y1[0][si, sj], ref) <= TOL[dtype]
    # integer operands, no activation: exact
    Ai = synth.integers(6100 + M, "A", M, K); Bi = synth.integers(6100 + M, "B", K, N)
    bi = synth.integers(6100 + M, "bias", 1, N, -5, 5)[0]
    Ais, Bis = store(Ai, dtype, False), store(Bi, dtype, bool(layout & 1))
    Yi, _, _ = run_gpu(Ais, Bis, bi, 1, M, N, K, dtype, synth.ACT_NONE, layout, variant=vid)
    refi = oracle.gemm_epilogue_sampled(sb, si, sj, Ais, Bis, bi, M, N, K, dtype=dtype, act=synth.ACT_NONE, layout=layout & 3)
    want = (synth.bf16_bits_to_f32(oracle.bf16_from_double(refi)).astype(np.float64) if dtype == BF16
            else oracle.f16_to_double(oracle.f16_from_double(refi)))
    assert np.array_equal(Yi[0][si, sj], want)


def test_the_dispatcher_takes_it_where_the_last_round_is_nearly_empty():
    P = 0x10000
    def chosen(M, N, K, layout=0):
        v = ob.optiml_select_variant(1, M, N, K, P, K, 0, P, K if layout & 1 else N, 0, P, 0, P, N, 0, layout, BF16, 0)
        return ob.optiml_variant_name(v)
    assert chosen(4352, 4352, 8192) == "xtail_split" and chosen(4352, 4352, 4352, 1) == "xtail_split"     # 17 x 17 tiles
    assert chosen(4096, 4096, 8192) != "xtail_split"                                    # 256 tiles: nothing left over
    assert chosen(8192, 8192, 8192) != "xtail_split"
    assert chosen(4352, 4352, 1024) != "xtail_split"                                    # too short a k to split
