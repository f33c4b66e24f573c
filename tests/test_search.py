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
    ev = analytic(fam, {"NS": 5, "PF": 1, "WN": 4, "PERSIST": 0})
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
    src = S.source(fam, {"NS": 4, "PF": 0, "WN": 4, "PERSIST": 1}, 1)
    assert "ringp::launch<ring::Cfg<4, true, false, 4>>" in src and 'extern "C" int cand_run' in src
    src = S.source(S.FAMILIES["skinny"], {"WN": 2, "WK": 4, "CG": 1, "NT": 1, "SPLIT": 0, "IL": 1}, 0)
    assert "skinny::skinny_launch<2, 4, 1, true, 0, true>" in src


def test_a_candidate_compiles_and_exports_its_entry_points():
    fam = S.FAMILIES["skinny"]
    path = S.build(fam, {"WN": 2, "WK": 4, "CG": 1, "NT": 1, "SPLIT": 0, "IL": 0}, 0)
    assert path is not None and os.path.exists(path)
    syms = subprocess.run(["nm", "-D", "--defined-only", path], capture_output=True, text=True, check=True).stdout
    assert " T cand_run" in syms and " T cand_resources" in syms


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
