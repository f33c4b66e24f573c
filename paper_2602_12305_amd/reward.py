"""Composite reward of the paper's search (section 3.2, "Reward Model"), used by the
variant sweep to score a kernel variant against a baseline variant.

    r_time  = tanh(alpha_t * (T0 - T) / max(T0, eps))                       (time reward)
    r_proxy = sum_{m in sm,dram,tex} w_m clip((SOL_m - SOL_m0)/100)
            + sum_{x in l1,dramB,inst} w_x clip((X0 - X)/(X0 + eps))         (proxy reward)
    p_guard = l_spill [scratch > 0] + l_regs [regs > rho_max] + l_work [dramB or inst inflated]
    R       = b_time r_time + b_proxy r_proxy + b_llm r_llm - p_guard         (total reward)

with clip(z) = max(-1, min(1, z)), bottleneck-aware weights from the appendix
"Bottleneck-aware proxy weighting" (memory-bound if SOL_dram - SOL_sm > delta,
compute-bound if SOL_sm - SOL_dram > delta, delta = 7.5; base weights, the regime
tables and the regression penalties are the paper's table of proxy-metric weights).
A candidate that fails its correctness tests gets -inf.

The profiler metrics are the MI355X analogues of the paper's Nsight Compute fields:
sol_sm = percent of the MFMA (or fp32 vector) roof reached, sol_dram = percent of the
HBM roof, sol_tex = percent of the L1/texture-path busy, l1 = L1 requests, dram_bytes =
HBM bytes, inst = executed instructions.

Readings where the paper is silent: alpha_t = 0.40 (its "time mixing" entry) is used as
the tanh sensitivity; beta_time = 1, beta_proxy = 0.25, beta_llm = 0 (no LLM judge here);
all guardrail lambdas = 1; rho_max = 512 registers per lane (the unified VGPR + AGPR file of
a CDNA SIMD at one wave, as hipFuncGetAttributes counts them); inflation threshold 1.5x.
A term that regresses is charged its regression penalty weight times the size of the
regression (on top of the negative progress term).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

EPS = 1e-12
ALPHA_T = 0.40
DELTA = 7.5
BETA_TIME, BETA_PROXY, BETA_LLM = 1.0, 0.25, 0.0
LAMBDA_SPILL = LAMBDA_REGS = LAMBDA_WORK = 1.0
RHO_MAX = 512
INFLATION = 1.5

# progress weights: sm, dram, tex, l1, dram_bytes, inst
W_BASE = {"sm": 0.20, "dram": 0.30, "tex": 0.10, "l1": 0.15, "dram_bytes": 0.15, "inst": 0.10}
W_MEMORY = {"sm": 0.20, "dram": 0.90, "tex": 0.10, "l1": 0.15, "dram_bytes": 0.45, "inst": 0.10}
W_COMPUTE = {"sm": 0.60, "dram": 0.30, "tex": 0.10, "l1": 0.15, "dram_bytes": 0.15, "inst": 0.30}
PENALTY = {"sm": 0.05, "dram": 0.05, "tex": 0.03, "l1": 0.04, "dram_bytes": 0.04, "inst": 0.03}


@dataclass
class Profile:
    """Time and profiler signals of one variant (the paper's node state (T, m))."""
    time: float                      # seconds (or any unit, the same for both profiles)
    sol_sm: float | None = None      # percent
    sol_dram: float | None = None
    sol_tex: float | None = None
    l1: float | None = None
    dram_bytes: float | None = None
    inst: float | None = None
    regs: int | None = None
    scratch_bytes: int | None = None
    correct: bool = True
    extra: dict = field(default_factory=dict)


def clip(z: float) -> float:
    return max(-1.0, min(1.0, z))


def regime(p: Profile) -> str:
    """Bottleneck class of a state from its SOL gap."""
    if p.sol_sm is None or p.sol_dram is None:
        return "mixed"
    if p.sol_dram - p.sol_sm > DELTA:
        return "memory"
    if p.sol_sm - p.sol_dram > DELTA:
        return "compute"
    return "mixed"


def weights(kind: str) -> dict:
    return {"memory": W_MEMORY, "compute": W_COMPUTE, "mixed": W_BASE}[kind]


def time_reward(t0: float, t: float) -> float:
    return math.tanh(ALPHA_T * (t0 - t) / max(t0, EPS))


def proxy_reward(base: Profile, cand: Profile) -> float:
    """Shaping term; metrics missing on either side contribute nothing."""
    w = weights(regime(base))
    total = 0.0
    for key, attr in (("sm", "sol_sm"), ("dram", "sol_dram"), ("tex", "sol_tex")):
        a, b = getattr(base, attr), getattr(cand, attr)
        if a is None or b is None:
            continue
        d = clip((b - a) / 100.0)
        total += w[key] * d
        if d < 0:
            total += PENALTY[key] * d
    for key, attr in (("l1", "l1"), ("dram_bytes", "dram_bytes"), ("inst", "inst")):
        a, b = getattr(base, attr), getattr(cand, attr)
        if a is None or b is None:
            continue
        d = clip((a - b) / (a + EPS))
        total += w[key] * d
        if d < 0:
            total += PENALTY[key] * d
    return total


def guard_penalty(base: Profile, cand: Profile) -> float:
    p = 0.0
    if cand.scratch_bytes is not None and cand.scratch_bytes > 0:
        p += LAMBDA_SPILL
    if cand.regs is not None and cand.regs > RHO_MAX:
        p += LAMBDA_REGS
    inflated = False
    for attr in ("dram_bytes", "inst"):
        a, b = getattr(base, attr), getattr(cand, attr)
        if a is not None and b is not None and a > 0 and b > INFLATION * a:
            inflated = True
    if inflated:
        p += LAMBDA_WORK
    return p


def total_reward(base: Profile, cand: Profile, r_llm: float = 0.0) -> float:
    if not cand.correct:
        return -math.inf
    return (BETA_TIME * time_reward(base.time, cand.time) + BETA_PROXY * proxy_reward(base, cand)
            + BETA_LLM * r_llm - guard_penalty(base, cand))


def keep(base: Profile, cand: Profile, min_gain: float = 0.01) -> bool:
    """Stand-in for the paper's judge verdict: correct, and faster than the baseline by more
    than the noise threshold."""
    return cand.correct and cand.time < base.time * (1.0 - min_gain)
