"""The sweep's score: values worked by hand from the paper's reward equations and weight table."""
import math

import pytest

from paper_2602_12305_amd import reward as R


def test_time_reward_values():
    assert R.time_reward(10.0, 10.0) == 0.0
    assert R.time_reward(10.0, 5.0) == pytest.approx(math.tanh(0.2))          # 0.4 * 0.5
    assert R.time_reward(10.0, 20.0) == pytest.approx(-math.tanh(0.4))
    assert R.time_reward(0.0, 1.0) < 0 and math.isfinite(R.time_reward(0.0, 1.0))
    assert R.time_reward(1.0, 1e9) >= -1.0 and R.time_reward(1.0, 0.0) == pytest.approx(math.tanh(0.4))


def test_regimes_follow_the_sol_gap_margin():
    assert R.regime(R.Profile(1, sol_sm=50, sol_dram=58)) == "memory"
    assert R.regime(R.Profile(1, sol_sm=50, sol_dram=57.5)) == "mixed"       # gap must exceed 7.5
    assert R.regime(R.Profile(1, sol_sm=71.26, sol_dram=8.42)) == "compute"  # the paper's matmul baseline row
    assert R.regime(R.Profile(1)) == "mixed"
    assert R.weights("memory")["dram"] == 0.90 and R.weights("memory")["dram_bytes"] == 0.45
    assert R.weights("compute")["sm"] == 0.60 and R.weights("compute")["inst"] == 0.30
    assert R.weights("mixed") == R.W_BASE and abs(sum(R.W_BASE.values()) - 1.0) < 1e-12
    # the emphasised entries are the base ones scaled by 3
    assert R.W_MEMORY["dram"] == pytest.approx(3 * R.W_BASE["dram"]) and R.W_COMPUTE["sm"] == pytest.approx(3 * R.W_BASE["sm"])


def test_proxy_reward_on_the_papers_matmul_rows():
    # Table 1, matmul: GPT 5.1 baseline vs full OptiML; baseline is compute-bound (71.26 vs 8.42)
    base = R.Profile(7.20, sol_sm=71.26, sol_dram=8.42, sol_tex=91.36, dram_bytes=63, l1=408, inst=419)
    cand = R.Profile(4.40, sol_sm=81.17, sol_dram=11.03, sol_tex=92.61, dram_bytes=70, l1=282, inst=381)
    want = (0.60 * (81.17 - 71.26) / 100 + 0.30 * (11.03 - 8.42) / 100 + 0.10 * (92.61 - 91.36) / 100
            + 0.15 * (408 - 282) / 408 + (0.15 + 0.04) * (63 - 70) / 63 + 0.30 * (419 - 381) / 419)
    assert R.proxy_reward(base, cand) == pytest.approx(want, rel=1e-12)
    assert R.guard_penalty(base, cand) == 0.0
    total = math.tanh(0.4 * (7.20 - 4.40) / 7.20) + 0.25 * want
    assert R.total_reward(base, cand) == pytest.approx(total, rel=1e-12)
    assert R.keep(base, cand)


def test_clip_and_missing_metrics():
    base = R.Profile(1.0, sol_sm=10, sol_dram=10, inst=100)
    cand = R.Profile(1.0, sol_sm=10, sol_dram=10, inst=1000)       # 9x more instructions: clipped at -1
    assert R.proxy_reward(base, cand) == pytest.approx(-(0.10 + 0.03))
    assert R.proxy_reward(R.Profile(1.0), R.Profile(1.0)) == 0.0
    assert R.clip(3) == 1 and R.clip(-3) == -1 and R.clip(0.25) == 0.25


def test_guardrails_and_rejection():
    base = R.Profile(1.0, dram_bytes=100, inst=100, regs=64, scratch_bytes=0)
    assert R.guard_penalty(base, R.Profile(1.0, scratch_bytes=16)) == 1.0
    assert R.guard_penalty(base, R.Profile(1.0, regs=513)) == 1.0
    assert R.guard_penalty(base, R.Profile(1.0, regs=512)) == 0.0
    assert R.guard_penalty(base, R.Profile(1.0, dram_bytes=151)) == 1.0
    assert R.guard_penalty(base, R.Profile(1.0, dram_bytes=150, inst=150)) == 0.0
    assert R.guard_penalty(base, R.Profile(1.0, dram_bytes=151, inst=151, regs=600, scratch_bytes=4)) == 3.0
    assert R.total_reward(base, R.Profile(0.5, correct=False)) == -math.inf
    assert not R.keep(base, R.Profile(0.995)) and not R.keep(base, R.Profile(0.5, correct=False))
    # a faster but spilling candidate scores below a slightly slower clean one
    assert R.total_reward(base, R.Profile(0.8, scratch_bytes=8)) < R.total_reward(base, R.Profile(0.9))
