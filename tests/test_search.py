"""Host logic of the tree search (paper section 3.2: UCT selection, reward back-up, KEEP chains)."""
import math
import os
import subprocess

import pytest

from paper_2602_12305_amd import reward as R
from paper_2602_12305_amd import search as S


def test_uct_value_and_unvisited_first():
    n = S.Node(params={}, visits=3, total=1.5)
    # Q + c sqrt(ln N_parent / N_child) = 0.5 + 1.4 sqrt(ln 10 / 3), worked by hand
    assert S.uct(n, 10, 1.4) == pytest.approx(0.5 + 1.4 * math.sqrt(2.302585092994046 / 3.0), rel=1e-12)
    assert S.uct(n, 10, 1.4) == pytest.approx(1.726522, abs=1e-6)      # sqrt(0.7675284) = 0.8760870
    assert S.uct(S.Node(params={}), 10) == math.inf
    # more visits at equal mean value -> smaller bonus
    assert S.uct(S.Node(params={}, visits=30, total=15.0), 100) < S.uct(S.Node(params={}, visits=3, total=1.5), 100)


@pytest.mark.parametrize("name", sorted(S.FAMILIES))
def test_edits_are_valid_single_steps_and_reversible(name):
    fam = S.FAMILIES[name]
    assert fam.valid(fam.root)
    pts = S.reachable(fam, fam.root, 3)
    assert len({S.key(p) for p in pts}) == len(pts) > 3
    for p in pts:
        assert fam.valid(p)
        for label, q in S.edits(fam, p):
            diff = [k for k in p if p[k] != q[k]]
            assert len(diff) == 1
            k = diff[0]
            assert abs(fam.domains[k].index(p[k]) - fam.domains[k].index(q[k])) == 1
            assert any(S.key(back) == S.key(p) for _, back in S.edits(fam, q))     # every edit can be undone


def analytic(fam, optimum, dead=()):
    """Time grows with the distance (in domain steps) from `optimum`; `dead` points fail their test."""
    def ev(p):
        d = sum(abs(fam.domains[k].index(p[k]) - fam.domains[k].index(optimum[k])) for k in p)
        return R.Profile(time=1.5 ** d, regs=64, scratch_bytes=0, correct=S.key(p) not in dead)
    return ev


def test_search_reaches_the_optimum_through_keep_edges():
    fam = S.FAMILIES["skinny"]
    opt = {"WN": 1, "WK": 4, "CG": 1, "NT": 0, "SPLIT": 1, "IL": 1}       # four edits from the root
    assert fam.valid(opt)
    root, nodes = S.search(fam, fam.root, analytic(fam, opt), budget=120, seed=1)
    best, path = S.best_keep_chain(root)
    assert S.key(best.params) == S.key(opt)
    assert path[0] is root and path[-1] is best
    times = [n.profile.time for n in path]
    assert all(b < a * 0.99 for a, b in zip(times, times[1:]))            # every step of the chain is a KEEP
    assert all(n.keep for n in path[1:])
    assert max(n.depth for n in nodes) <= S.MAX_DEPTH
    # the same seed gives the same tree
    root2, nodes2 = S.search(fam, fam.root, analytic(fam, opt), budget=120, seed=1)
    assert [S.key(n.params) for n in nodes] == [S.key(n.params) for n in nodes2]


def test_budget_counts_distinct_kernels_and_visits_add_up():
    fam = S.FAMILIES["ring_bf16"]
    calls = []
    ev = analytic(fam, {"NS": 5, "PF": 1, "WN": 4, "PERSIST": 0, "BAND": 8, "SWZ": 4})
    root, nodes = S.search(fam, fam.root, lambda p: (calls.append(S.key(p)), ev(p))[1], budget=7, seed=0)
    assert len(calls) == len(set(calls)) == 8             # the root plus `budget` kernels, each measured once
    assert len(nodes) >= 8 and root.visits == len(nodes) - 1
    for n in nodes:
        assert n.visits >= sum(ch.visits for ch in n.children)
        if n.parent is not None and n.alive:
            assert n.reward == pytest.approx(R.total_reward(n.parent.profile, n.profile))


def test_dead_candidates_are_scored_as_failures_and_never_expanded():
    fam = S.FAMILIES["ring_f32"]
    dead = {S.key({"BM": 256, "NS": 4}), S.key({"BM": 128, "NS": 5})}
    root, nodes = S.search(fam, fam.root, analytic(fam, {"BM": 256, "NS": 3}, dead), budget=50, seed=3)
    for n in nodes:
        if S.key(n.params) in dead:
            assert not n.alive and not n.children and not n.untried and not n.keep
            assert n.reward == -math.inf and n.total == pytest.approx(S.FAIL_REWARD * n.visits)
    best, path = S.best_keep_chain(root)
    assert all(S.key(n.params) not in dead for n in path)
    assert S.key(best.params) == S.key({"BM": 256, "NS": 3})      # reached around the dead node: 128/4 -> 128/3 -> 256/3


def test_depth_limit():
    fam = S.FAMILIES["skinny"]
    root, nodes = S.search(fam, fam.root, analytic(fam, {"WN": 8, "WK": 2, "CG": 1, "NT": 0, "SPLIT": 8, "IL": 0}), budget=300,
                           depth=2, seed=0)
    assert max(n.depth for n in nodes) == 2
    assert all(not n.untried for n in nodes if n.depth == 2)


def test_candidate_source_names_the_instantiation():
    fam = S.FAMILIES["ring_bf16"]
    src = S.source(fam, {"NS": 4, "PF": 0, "WN": 4, "PERSIST": 1, "BAND": 8, "SWZ": 4}, 1)
    assert "ringp::launch<ring::Cfg<4, true, false, 4, DT_BF16, 0, false, 8, 4>>" in src and 'extern "C" int cand_run' in src
    # the tile walk and the LDS swizzle key are edit classes of this family; the persistent kernel keeps its own
    assert any(lbl.startswith("BAND:") for lbl, _ in S.edits(fam, fam.root)) and any(lbl.startswith("SWZ:") for lbl, _ in S.edits(fam, fam.root))
    assert not fam.valid({"NS": 4, "PF": 0, "WN": 4, "PERSIST": 1, "BAND": 4, "SWZ": 4})
    src = S.source(S.FAMILIES["skinny"], {"WN": 2, "WK": 4, "CG": 1, "NT": 1, "SPLIT": 0, "IL": 1}, 0)
    assert "skinny::skinny_launch<2, 4, 1, true, 0, true>" in src


def test_a_candidate_compiles_and_exports_its_entry_points():
    fam = S.FAMILIES["skinny"]
    path = S.build(fam, {"WN": 2, "WK": 4, "CG": 1, "NT": 1, "SPLIT": 0, "IL": 0}, 0)
    assert path is not None and os.path.exists(path)
    syms = subprocess.run(["nm", "-D", "--defined-only", path], capture_output=True, text=True, check=True).stdout
    assert " T cand_run" in syms and " T cand_resources" in syms


def test_profiler_signals_from_counters():
    # the bf16 8192^3 kernel's counters: 1.0737e9 matrix-pipe busy cycles over 1024 SIMDs against 1.1317e7 / 8 active
    # cycles per XCD -> 74.1 % busy; 806 645 KiB fetched (x 2) + 131 072 KiB written in 0.8323 ms -> 26.0 % of 8 TB/s
    c = {"SQ_VALU_MFMA_BUSY_CYCLES": 1.0737e9, "GRBM_GUI_ACTIVE": 1.1317e7, "FETCH_SIZE": 806645.0, "WRITE_SIZE": 131072.0,
         "TCP_TOTAL_CACHE_ACCESSES_sum": 5.0e8, "SQ_INSTS_VALU": 6.19e7, "SQ_INSTS_SALU": 3.87e7, "SQ_INSTS_LDS": 3.40e7,
         "SQ_INSTS_VMEM_RD": 8.4e6, "SQ_INSTS_VMEM_WR": 1.0e6}
    sig = S.signals(c, 0.8323e-3)
    assert sig["sol_sm"] == pytest.approx(74.12, abs=0.02)
    assert sig["dram_bytes"] == pytest.approx((2 * 806645.0 + 131072.0) * 1024.0)
    assert sig["sol_dram"] == pytest.approx(100.0 * sig["dram_bytes"] / 0.8323e-3 / 8e12, rel=1e-12) and 26.0 < sig["sol_dram"] < 27.0
    assert sig["l1"] == 5.0e8 and sig["inst"] == pytest.approx(6.19e7 + 3.87e7 + 3.40e7 + 8.4e6 + 1.0e6)
    assert S.signals({}, 1e-3) == {"sol_sm": None, "sol_dram": None, "l1": None, "dram_bytes": None, "inst": None}
    # every counter group stays inside what one rocprofv3 run can hold
    for g in S.PMC_GROUPS:
        assert sum(n.startswith("SQ_") for n in g) <= 8 and sum(n.startswith("TCP_") for n in g) <= 4
        assert 3 * ("FETCH_SIZE" in g) + 2 * ("WRITE_SIZE" in g) <= 4 and sum(n.startswith("GRBM_") for n in g) <= 2


def test_counters_of_the_dominant_kernel_are_read_from_the_profilers_csv(tmp_path):
    f = tmp_path / "r_counter_collection.csv"
    rows = ["Kernel_Name,Counter_Name,Counter_Value",
            '"void optiml::skinny::skinny_kernel<1>(P)",FETCH_SIZE,1000', '"void optiml::skinny::skinny_kernel<1>(P)",FETCH_SIZE,1200',
            '"void optiml::skinny::skinny_reduce_kernel(P)",FETCH_SIZE,16', '"void optiml::copy_kernel(a)",FETCH_SIZE,99999',
            '"at::native::fill(x)",FETCH_SIZE,88888', '"void optiml::skinny::skinny_kernel<1>(P)",WRITE_SIZE,7']
    f.write_text("\n".join(rows) + "\n")
    got = S.main_kernel_counters([str(f)], ("FETCH_SIZE", "WRITE_SIZE", "SQ_INSTS_VALU"))
    assert got == {"FETCH_SIZE": 1100.0, "WRITE_SIZE": 7.0}


def test_measured_signals_drive_the_regime_the_proxy_terms_and_the_guardrail():
    """With profiler signals in the node state the reward is more than a function of time: the regime follows the
    measured SOL gap, a candidate that moves fewer bytes is preferred at equal time, and one that moves 1.6 times the
    bytes pays the work-inflation penalty (paper section 3.2, proxy reward and guardrails)."""
    base = R.Profile(time=1.0, sol_sm=20.0, sol_dram=70.0, l1=1e6, dram_bytes=1e9, inst=1e7, regs=128, scratch_bytes=0)
    lean = R.Profile(time=1.0, sol_sm=20.0, sol_dram=70.0, l1=1e6, dram_bytes=0.8e9, inst=1e7, regs=128, scratch_bytes=0)
    fat = R.Profile(time=1.0, sol_sm=20.0, sol_dram=70.0, l1=1e6, dram_bytes=1.6e9, inst=1e7, regs=128, scratch_bytes=0)
    blind = R.Profile(time=1.0, regs=128, scratch_bytes=0)
    assert R.regime(base) == "memory" and R.regime(blind) == "mixed"
    assert R.proxy_reward(base, lean) == pytest.approx(R.W_MEMORY["dram_bytes"] * 0.2)
    assert R.total_reward(base, lean) == pytest.approx(0.25 * 0.45 * 0.2) and R.total_reward(base, lean) > R.total_reward(base, base)
    assert R.guard_penalty(base, fat) == 1.0 and R.total_reward(base, fat) < -1.0
    assert R.proxy_reward(blind, blind) == 0.0 and R.total_reward(blind, blind) == 0.0       # no counters: time only


@pytest.mark.gpu
def test_profiled_search_carries_measured_signals_into_the_reward(tmp_path):
    """The search as a program of its own (it must not share a process with anything that uses the GPU): the root and
    two edits of the streaming family on the 256^3 workload, each timed by the worker child and profiled by three
    rocprofv3 counter passes.  Every node's state then holds measured SOL percentages, bytes and instruction counts,
    and the children's rewards contain a proxy term that is not zero."""
    import json
    import sys
    out = tmp_path / "search.jsonl"
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-m", "paper_2602_12305_amd.search", "--workload", "c1_f32_256_relu", "--family", "skinny",
                        "--budget", "2", "--pmc", "--steps", "5", "--warmup", "2", "--out", str(out)],
                       cwd=root, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    recs = [json.loads(l) for l in open(out)]
    assert len(recs) >= 3 and recs[0]["edit"] == "root"
    for j in recs:
        assert j["correct"], j
        assert j["sol_sm"] is not None and j["sol_dram"] is not None and 0.0 <= j["sol_sm"] <= 100.0 and 0.0 < j["sol_dram"] <= 100.0
        assert j["dram_bytes"] > 0 and j["inst"] > 0 and j["l1"] > 0 and j["regime"] in ("memory", "compute", "mixed")
        assert j["counters"]["FETCH_SIZE"] > 0 and j["counters"]["SQ_INSTS_VALU"] > 0
    assert any(abs(j["r_proxy"]) > 0.0 for j in recs[1:])
    for j in recs[1:]:
        assert j["reward"] == pytest.approx(j["r_time"] + 0.25 * j["r_proxy"] - j["p_guard"], abs=2e-4)


@pytest.mark.gpu
def test_the_searchs_best_candidate_agrees_with_the_oracle():
    """What the search would hand back as the new default is checked against the CPU oracle, not only against the
    fallback kernel the search itself uses: the end of the best KEEP chain on the 256^3 workload, every output entry."""
    import ctypes

    import numpy as np
    import torch

    import oracle
    from inputs import synth
    fam = S.FAMILIES["skinny"]
    ev = S.Evaluator("c1_f32_256_relu", fam, steps=5, warmup=2)
    root, nodes = S.search(fam, fam.root, ev, budget=4, seed=1)
    best, _ = S.best_keep_chain(root)
    lib = ctypes.CDLL(S.build(fam, best.params, 0))
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    lib.cand_run.argtypes = [i64, i64, i64, i64, vp, i64, i64, vp, i64, i64, vp, i64, vp, i64, i64, ci, ci, ci, vp]
    lib.cand_run.restype = ci
    C = ev.r.new_c()
    assert ev._call(lib.cand_run, C) == 0
    torch.cuda.synchronize()
    w = synth.make_workload("c1_f32_256_relu")
    ref = oracle.gemm_epilogue(w.A, w.B, w.bias, w.M, w.N, w.K, dtype=w.dtype, act=w.act, layout=w.layout)[0]
    got = C.cpu().numpy().reshape(ref.shape).astype(np.float64)
    rho = float(np.sqrt(np.mean(ref * ref)))
    assert float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rho))) <= 1e-5


@pytest.mark.gpu
def test_search_runs_on_the_gpu_and_every_candidate_passes_its_check():
    """Four kernels of the streaming family on the 256^3 workload: each is compiled (or found in the
    cache), loaded next to the library, compared with the fallback kernel and timed."""
    fam = S.FAMILIES["skinny"]
    ev = S.Evaluator("c1_f32_256_relu", fam, steps=5, warmup=2)
    root, nodes = S.search(fam, fam.root, ev, budget=3, seed=0)
    assert len({S.key(n.params) for n in nodes}) == 4
    for n in nodes:
        assert n.alive and n.profile.correct and n.profile.extra["err"] <= 2e-5
        assert 0 < n.profile.time < 1e-3 and n.profile.regs > 0 and n.profile.scratch_bytes == 0
    best, path = S.best_keep_chain(root)
    assert best.profile.time <= root.profile.time
