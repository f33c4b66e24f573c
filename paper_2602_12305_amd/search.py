"""Tree search over kernel-template parameters: the paper's search loop without its LLM steps.

    python -m paper_2602_12305_amd.search --workload c2_f32_skinny16_silu --family skinny \
        --budget 24 [--depth 6] [--c 1.4] [--seed 0] [--out search.jsonl]
    python -m paper_2602_12305_amd.search --family skinny --prebuild 2      # compile only, no GPU

The paper (section 3.2, equations for UCT and for the rewards, and its algorithm box)
searches a tree whose nodes are kernels and whose edges are edits proposed by a language
model; every node is compiled, tested, profiled and scored, the score is backed up the
path, and the answer is the end of the best chain of KEEP verdicts.  Here the proposer is
replaced by the finite set of single-parameter edits of a kernel template (tile shape, ring
depth, prefetch, wave layout, split-K, k interleaving, non-temporal hint, persistence); everything else is
the paper's loop:

  * selection by UCT, Q + c sqrt(ln N_parent / N_child), c = 1.4, depth limit 6;
  * expansion by one untried edit; the new kernel is a template instantiation compiled into
    a small shared library of its own (cached under csrc/_cand/) and loaded next to the main
    library;
  * evaluation: output compared with the guarded fallback kernel on 65,536 seeded entries and
    a bitwise repeat (a failing, unsupported or uncompilable candidate is a dead node with
    the paper's failure score), HIP-event timing, registers / scratch / LDS from
    hipFuncGetAttributes;
  * reward of a node relative to its parent: the composite reward of
    paper_2602_12305_amd.reward (time term plus proxy terms minus guardrails);
  * KEEP = correct and faster than the parent by more than 1 %; the result is the fastest
    node reachable from the root through KEEP edges only.

Nodes with equal parameters reached along different paths share one measurement.

With --pmc every correct candidate is also PROFILED, as the paper profiles every node (its node
state is (T, m) with m the profiler's metric vector): three rocprofv3 counter passes per distinct
kernel, each a child process of its own (separate from timing, as the paper runs its profiler),
give HBM bytes, L1 requests, executed instructions and matrix-pipe busy cycles; from them the
node's SOL percentages are MEASURED (matrix pipe busy share of the launch, HBM bytes over time
against 8 TB/s), so the bottleneck regime and the proxy terms of the reward come from counters and
the traffic / instruction inflation guardrail can fire.  In that mode this process never touches
the GPU: a worker child times and checks the candidates, the counter passes are further children.
Without --pmc the SOL terms are left out (the proxy reward is then 0 rather than a second function
of the time).
"""
from __future__ import annotations

import argparse
import concurrent.futures as cf
import ctypes
import hashlib
import json
import math
import os
import random
import subprocess
import sys
from dataclasses import dataclass, field

from . import reward as R

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
CAND = os.path.join(CSRC, "_cand")
FAIL_REWARD = -1.0          # finite stand-in for the paper's -inf when averaging over visits
UCT_C = 1.4
MAX_DEPTH = 6


# ---------------------------------------------------------------------------------------------
# kernel families: parameter domains, validity, and how a point becomes C++

@dataclass(frozen=True)
class Family:
    name: str
    header: str
    domains: dict                 # parameter -> ordered list of values
    valid: object                 # dict -> bool
    exprs: object                 # (dict, layout) -> (supports, launch, kernel) C++ expressions
    root: dict                    # the library's default point


def _skinny_exprs(p, layout):
    t = f"{p['WN']}, {p['WK']}, {p['CG']}, {'true' if p['NT'] else 'false'}"
    il = "true" if p["IL"] else "false"
    return ("skinny::skinny_supports", f"skinny::skinny_launch<{t}, {p['SPLIT']}, {il}>",
            f"skinny::skinny_kernel<{t}, {il}>")


def _skinny_dma_exprs(p, layout):
    t = f"{p['WK']}, {p['CG']}, {p['NS']}, {'true' if p['NT'] else 'false'}"
    return ("skinny::skinny_dma_supports", f"skinny::skinny_dma_launch<{t}>", f"skinny::skinny_dma_kernel<{t}>")


def _skinny16_exprs(dt):
    def exprs(p, layout):
        t = f"{p['WN']}, {p['WK']}, {p['CG']}, {'true' if p['NT'] else 'false'}"
        il = "true" if p["IL"] else "false"
        return (f"skinny16::supports<{dt}>", f"skinny16::launch<{dt}, {t}, {p['SPLIT']}, {il}>",
                f"skinny16::skinny16_kernel<{dt}, {t}, {il}>")
    return exprs


def _ringf_exprs(p, layout):
    c = f"ringf::Cfg<{p['BM']}, {p['NS']}, {'true' if layout & 1 else 'false'}>"
    return (f"ringf::supports<{c}>", f"ringf::launch<{c}>", f"ringf::gemm_ring_f32_kernel<{c}>")


def _ring_exprs(p, layout):
    c = (f"ring::Cfg<{p['NS']}, {'true' if layout & 1 else 'false'}, {'true' if p['PF'] else 'false'}, {p['WN']}, DT_BF16, 0, false, "
         f"{p['BAND']}, {p['SWZ']}>")
    if p["PERSIST"]:
        return (f"ringp::supports<{c}>", f"ringp::launch<{c}>", f"ringp::gemm_ring_persistent_kernel<{c}>")
    return (f"ring::supports<{c}>", f"ring::launch<{c}>", f"ring::gemm_ring_kernel<{c}>")


FAMILIES = {
    "skinny": Family(
        "skinny", "kernel_skinny.hpp",
        {"WN": [1, 2, 4, 8], "WK": [1, 2, 4, 8, 16], "CG": [1, 2], "NT": [0, 1], "SPLIT": [0, 1, 2, 4, 8], "IL": [0, 1]},
        lambda p: p["WN"] * p["WK"] <= 16 and not (p["WN"] * p["WK"] > 8 and p["CG"] > 1),
        _skinny_exprs, {"WN": 1, "WK": 8, "CG": 2, "NT": 1, "SPLIT": 0, "IL": 1}),
    # fp32 streaming kernels with B staged through LDS by direct loads: WK waves x NS stages of 1 + 4 CG KiB fit
    # the 160 KiB of LDS, and the counted wait ((NS - 1) x (1 + 4 CG) loads outstanding) has six bits
    "skinny_dma": Family(
        "skinny_dma", "kernel_skinny.hpp",
        {"WK": [2, 4, 8], "CG": [1, 2, 4], "NS": [2, 3, 4, 6, 8], "NT": [0, 1]},
        lambda p: p["WK"] * p["NS"] * (1 + 4 * p["CG"]) <= 160 and (p["NS"] - 1) * (1 + 4 * p["CG"]) < 64,
        _skinny_dma_exprs, {"WK": 4, "CG": 2, "NS": 2, "NT": 1}),
    # 16-bit streaming kernels: the cross-wave reduction buffer (WK x 16 rows x 128 CG WN columns of
    # fp32) must fit 64 KiB of static LDS
    "skinny16_bf16": Family(
        "skinny16_bf16", "kernel_skinny16.hpp",
        {"WN": [1, 2, 4, 8], "WK": [1, 2, 4, 8, 16], "CG": [1, 2], "NT": [0, 1], "SPLIT": [0, 1, 2, 4, 8], "IL": [0, 1]},
        lambda p: p["WN"] * p["WK"] <= 16 and not (p["WN"] * p["WK"] > 8 and p["CG"] > 1)
        and (p["WK"] == 1 or p["WK"] * p["CG"] * p["WN"] <= 8),
        _skinny16_exprs("DT_BF16"), {"WN": 1, "WK": 4, "CG": 2, "NT": 1, "SPLIT": 0, "IL": 1}),
    "ring_f32": Family(
        "ring_f32", "kernel_ring_f32.hpp",
        {"BM": [128, 256], "NS": [3, 4, 5, 6]},
        lambda p: p["NS"] * (p["BM"] + 128) * 64 <= 160 * 1024,
        _ringf_exprs, {"BM": 128, "NS": 4}),
    "ring_bf16": Family(
        "ring_bf16", "kernel_ring_persistent.hpp",
        # BAND: tile rows per band of the workgroup -> tile walk (which panels an XCD's L2 shares);
        # SWZ: XOR key step of the row-major B tile in LDS (which banks a transposing read touches)
        {"NS": [3, 4, 5], "PF": [0, 1], "WN": [2, 4], "PERSIST": [0, 1], "BAND": [2, 4, 8, 16], "SWZ": [2, 4]},
        lambda p: (not p["PF"] or p["NS"] >= 4)
        and (not p["PERSIST"] or (p["NS"] * 32768 + 2 * p["WN"] * 1024 <= 160 * 1024 and p["BAND"] == 8 and p["SWZ"] == 4)),
        _ring_exprs, {"NS": 4, "PF": 1, "WN": 4, "PERSIST": 0, "BAND": 8, "SWZ": 4}),
}


def key(params: dict) -> str:
    return "_".join(f"{k.lower()}{v}" for k, v in sorted(params.items()))


def edits(fam: Family, params: dict):
    """Single-parameter moves to a neighbouring value of the domain that stay valid."""
    out = []
    for k, dom in fam.domains.items():
        i = dom.index(params[k])
        for j in (i - 1, i + 1):
            if 0 <= j < len(dom):
                q = dict(params)
                q[k] = dom[j]
                if fam.valid(q):
                    out.append((f"{k}:{params[k]}->{dom[j]}", q))
    return out


# ---------------------------------------------------------------------------------------------
# candidates as shared libraries

SOURCE = """// generated by paper_2602_12305_amd/search.py: one kernel-template instantiation behind a C ABI
#include "{header}"
using namespace optiml;
extern "C" int cand_run(int64_t batch, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, int64_t strideA,
                        const void *B, int64_t ldb, int64_t strideB, const float *bias, int64_t strideBias, void *C,
                        int64_t ldc, int64_t strideC, int layout, int dtype, int act, void *stream)
{{
    Problem p;
    p.batch = batch; p.M = M; p.N = N; p.K = K;
    p.A = A; p.lda = lda; p.strideA = batch > 1 ? strideA : 0;
    p.B = B; p.ldb = ldb; p.strideB = batch > 1 ? strideB : 0;
    p.bias = bias; p.strideBias = batch > 1 ? strideBias : 0;
    p.C = C; p.ldc = ldc; p.strideC = batch > 1 ? strideC : 0;
    p.layout = layout; p.dtype = dtype; p.act = act;
    if (!{supports}(p)) return -2;
    return {launch}(p, static_cast<hipStream_t>(stream)) == hipSuccess ? 0 : -3;
}}
extern "C" int cand_resources(int *regs, int *scratch, int *lds)
{{
    hipFuncAttributes a;
    if (hipFuncGetAttributes(&a, reinterpret_cast<const void *>(&{kernel})) != hipSuccess) return -3;
    *regs = a.numRegs; *scratch = (int)a.localSizeBytes; *lds = (int)a.sharedSizeBytes;
    return 0;
}}
"""

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wno-unused-function",
               "-Wno-inline-asm", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def source(fam: Family, params: dict, layout: int) -> str:
    s, l, k = fam.exprs(params, layout)
    return SOURCE.format(header=fam.header, supports=s, launch=l, kernel=k)


def lib_path(fam: Family, params: dict, layout: int) -> str:
    src = source(fam, params, layout)
    deps = "".join(open(os.path.join(CSRC, f)).read() for f in sorted(os.listdir(CSRC)) if f.endswith(".hpp"))
    h = hashlib.sha256((src + deps).encode()).hexdigest()[:12]
    return os.path.join(CAND, f"{fam.name}_l{layout}_{key(params)}_{h}.so")


def build(fam: Family, params: dict, layout: int) -> str | None:
    """Compile the candidate (if its library is not cached); None if the compiler rejects it."""
    out = lib_path(fam, params, layout)
    if os.path.exists(out):
        return out
    os.makedirs(CAND, exist_ok=True)
    cpp = out[:-3] + ".hip"
    with open(cpp, "w") as f:
        f.write(source(fam, params, layout))
    cmd = ["hipcc", *HIPCC_FLAGS, "-I", CSRC, "-I", os.path.join(HERE, "..", "include"), cpp, "-o", out + ".tmp",
           "-L", CSRC, "-loptiml", "-Wl,-rpath,$ORIGIN/..", "-Wl,-Bsymbolic"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(f"# compile failed for {fam.name} {params}:\n{r.stderr[-2000:]}\n")
        return None
    os.replace(out + ".tmp", out)
    return out


def reachable(fam: Family, root: dict, depth: int):
    seen, frontier = {key(root): root}, [root]
    for _ in range(depth):
        nxt = []
        for p in frontier:
            for _, q in edits(fam, p):
                if key(q) not in seen:
                    seen[key(q)] = q
                    nxt.append(q)
        frontier = nxt
    return list(seen.values())


# ---------------------------------------------------------------------------------------------
# the tree

@dataclass
class Node:
    params: dict
    parent: "Node | None" = None
    edit: str = "root"
    depth: int = 0
    profile: R.Profile | None = None
    alive: bool = True
    visits: int = 0
    total: float = 0.0
    reward: float = 0.0           # of this node relative to its parent
    keep: bool = False
    children: list = field(default_factory=list)
    untried: list = field(default_factory=list)

    @property
    def q(self):
        return self.total / self.visits if self.visits else 0.0


def uct(child: Node, parent_visits: int, c: float = UCT_C) -> float:
    """Upper confidence bound of the paper's selection rule; an unvisited child comes first."""
    if child.visits == 0:
        return math.inf
    return child.q + c * math.sqrt(math.log(max(parent_visits, 1)) / child.visits)


def search(fam: Family, root_params: dict, evaluate, budget: int, depth: int = MAX_DEPTH, c: float = UCT_C,
           seed: int = 0, log=None):
    """evaluate(params) -> reward.Profile (correct=False for a dead candidate).  `budget` counts the
    kernels evaluated beyond the root (a node whose parameters were measured before costs nothing);
    the number of iterations is capped at 50 times that.  Returns (root, nodes)."""
    rng = random.Random(seed)
    cache = {}

    def measured(params):
        k = key(params)
        if k not in cache:
            cache[k] = evaluate(params)
        return cache[k]

    def make(params, parent, edit):
        n = Node(params=params, parent=parent, edit=edit, depth=parent.depth + 1 if parent else 0)
        n.profile = measured(params)
        n.alive = bool(n.profile.correct)
        n.untried = edits(fam, params) if n.alive and n.depth < depth else []
        rng.shuffle(n.untried)
        if parent is not None:
            n.reward = R.total_reward(parent.profile, n.profile) if n.alive else -math.inf
            n.keep = n.alive and R.keep(parent.profile, n.profile)
        return n

    root = make(dict(root_params), None, "root")
    nodes = [root]
    if log:
        log(root)
    for _ in range(50 * budget):
        if len(cache) > budget:
            break
        node = root
        while not node.untried and node.children:          # selection
            live = [ch for ch in node.children if ch.alive] or node.children
            node = max(live, key=lambda ch: uct(ch, node.visits, c))
        if node.untried:                                   # expansion + evaluation
            edit, params = node.untried.pop()
            child = make(params, node, edit)
            node.children.append(child)
            nodes.append(child)
            if log:
                log(child)
            node = child
        r = node.reward if node.parent is not None else 0.0
        r = FAIL_REWARD if r == -math.inf else r
        while node is not None:                            # backpropagation
            node.visits += 1
            node.total += r
            node = node.parent
        if not any(n.untried for n in nodes if n.alive):
            break
    return root, nodes


def best_keep_chain(root: Node):
    """Fastest node reachable from the root through KEEP edges only, with its path."""
    best, stack = root, [root]
    while stack:
        n = stack.pop()
        if n.profile.time < best.profile.time:
            best = n
        stack.extend(ch for ch in n.children if ch.keep)
    path, n = [], best
    while n is not None:
        path.append(n)
        n = n.parent
    return best, path[::-1]


# ---------------------------------------------------------------------------------------------
# GPU evaluation

class Evaluator:
    def __init__(self, workload: str, fam: Family, steps: int, warmup: int, with_reference: bool = True):
        from .sweep import Runner
        from inputs import synth
        self.r = Runner(workload)
        self.fam, self.steps, self.warmup = fam, steps, warmup
        w, np = self.r.w, self.r.np
        if not with_reference:          # a counter pass: nothing but the candidate's own kernels may run
            return
        self.idx = synth.sample_entries(w.seed, 65536, w.batch, w.M, w.N)
        Cref = self.r.new_c()
        self.r.run(0, Cref)                                  # guarded fallback kernel
        self.r.torch.cuda.synchronize()
        self.ref = self.r.values(Cref, self.idx)
        self.rho = float(np.sqrt(np.mean(self.ref * self.ref))) or 1.0
        self.tol = 2e-5 if w.dtype == 0 else 2e-2

    def _call(self, fn, C):
        w, r = self.r.w, self.r
        P = lambda t: ctypes.c_void_p(t.data_ptr())
        return fn(w.batch, w.M, w.N, w.K, P(r.A), r.lda, r.sA, P(r.B), r.ldb, r.sB, P(r.bias), r.sBias, P(C), w.N,
                  w.M * w.N, w.layout, w.dtype, w.act, ctypes.c_void_p(r.torch.cuda.current_stream().cuda_stream))

    def __call__(self, params) -> R.Profile:
        r, w, np, torch = self.r, self.r.w, self.r.np, self.r.torch
        path = build(self.fam, params, w.layout)
        if path is None:
            return R.Profile(time=math.inf, correct=False, extra={"why": "compile"})
        lib = ctypes.CDLL(path)
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        lib.cand_run.argtypes = [i64, i64, i64, i64, vp, i64, i64, vp, i64, i64, vp, i64, vp, i64, i64, ci, ci, ci, vp]
        lib.cand_run.restype = ci
        C1, C2 = r.new_c(), r.new_c()
        st = self._call(lib.cand_run, C1)
        if st != 0:
            return R.Profile(time=math.inf, correct=False, extra={"why": f"status {st}"})
        self._call(lib.cand_run, C2)
        torch.cuda.synchronize()
        got = r.values(C1, self.idx)
        err = float(np.max(np.abs(got - self.ref) / np.maximum(np.abs(self.ref), self.rho)))
        correct = bool(err <= self.tol and torch.equal(C1, C2) and np.all(np.isfinite(got)))
        for _ in range(self.warmup):
            self._call(lib.cand_run, C1)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(self.steps):
            self._call(lib.cand_run, C1)
        e1.record()
        torch.cuda.synchronize()
        t = e0.elapsed_time(e1) / self.steps * 1e-3
        regs, scr, lds = ci(), ci(), ci()
        lib.cand_resources(ctypes.byref(regs), ctypes.byref(scr), ctypes.byref(lds))
        tfl, gbs = w.flops / t / 1e12, w.algorithmic_bytes / t / 1e9
        # the SOL fields stay empty here: they are the profiler's (see ProfiledEvaluator), and filling them from the
        # time alone would make the proxy reward a second function of the time
        return R.Profile(time=t, regs=regs.value, scratch_bytes=scr.value, correct=correct,
                         extra={"err": err, "lds": lds.value, "TFLOP/s": tfl, "GB/s": gbs})

    def launch_only(self, params, times=3):
        """A few launches of one candidate and nothing else: what a counter pass profiles."""
        path = build(self.fam, params, self.r.w.layout)
        lib = ctypes.CDLL(path)
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        lib.cand_run.argtypes = [i64, i64, i64, i64, vp, i64, i64, vp, i64, i64, vp, i64, vp, i64, i64, ci, ci, ci, vp]
        lib.cand_run.restype = ci
        C = self.r.new_c()
        for _ in range(times):
            self._call(lib.cand_run, C)
        self.r.torch.cuda.synchronize()


# ---------------------------------------------------------------------------------------------
# profiled evaluation: timing in a worker child, counters in rocprofv3 children

# One rocprofv3 run cannot split counters over passes: each group stays within the per-block limits
# (TCC: FETCH_SIZE takes 3 of 4, WRITE_SIZE 2; SQ: 8; TCP: 4; GRBM: 2).
PMC_GROUPS = (
    ("FETCH_SIZE",),
    ("WRITE_SIZE", "TCP_TOTAL_CACHE_ACCESSES_sum", "TCP_TCC_READ_REQ_sum"),
    ("SQ_INSTS_VALU", "SQ_INSTS_SALU", "SQ_INSTS_LDS", "SQ_INSTS_VMEM_RD", "SQ_INSTS_VMEM_WR", "SQ_VALU_MFMA_BUSY_CYCLES",
     "GRBM_GUI_ACTIVE"),
)
# what the byte counters read for a plain copy of known size on this chip (KiB -> bytes)
FETCH_SCALE, WRITE_SCALE = 2.0 * 1024.0, 1.0 * 1024.0
PEAK_HBM_BYTES_PER_S = 8.0e12
SIMDS, XCDS = 1024, 8


def signals(counters: dict, seconds: float) -> dict:
    """Profiler signals of the reward from raw per-dispatch counter sums and the kernel's time: SOL of the
    matrix pipe (busy cycles per SIMD over the launch's cycles per XCD), SOL of HBM (bytes over time against
    the peak), HBM bytes, L1 requests, executed instructions.  Missing counters give None."""
    out = {"sol_sm": None, "sol_dram": None, "l1": None, "dram_bytes": None, "inst": None}
    if "SQ_VALU_MFMA_BUSY_CYCLES" in counters and counters.get("GRBM_GUI_ACTIVE", 0) > 0:
        out["sol_sm"] = 100.0 * (counters["SQ_VALU_MFMA_BUSY_CYCLES"] / SIMDS) / (counters["GRBM_GUI_ACTIVE"] / XCDS)
    if "FETCH_SIZE" in counters and "WRITE_SIZE" in counters:
        out["dram_bytes"] = counters["FETCH_SIZE"] * FETCH_SCALE + counters["WRITE_SIZE"] * WRITE_SCALE
        if seconds > 0 and math.isfinite(seconds):
            out["sol_dram"] = 100.0 * out["dram_bytes"] / seconds / PEAK_HBM_BYTES_PER_S
    if "TCP_TOTAL_CACHE_ACCESSES_sum" in counters:
        out["l1"] = counters["TCP_TOTAL_CACHE_ACCESSES_sum"]
    inst = [counters[k] for k in ("SQ_INSTS_VALU", "SQ_INSTS_SALU", "SQ_INSTS_LDS", "SQ_INSTS_VMEM_RD", "SQ_INSTS_VMEM_WR")
            if k in counters]
    if len(inst) == 5:
        out["inst"] = float(sum(inst))
    return out


def main_kernel_counters(csv_paths, wanted) -> dict:
    """Mean per dispatch of each wanted counter for the library kernel that dominates the run: per kernel name
    the mean over its dispatches, then per counter the largest of those means (the copy kernel and
    framework kernels are left out)."""
    import csv
    per_kernel = {}
    for f in csv_paths:
        for row in csv.DictReader(open(f)):
            k = row["Kernel_Name"]
            if "optiml" not in k or "copy_kernel" in k:
                continue
            per_kernel.setdefault(k, {}).setdefault(row["Counter_Name"], []).append(float(row["Counter_Value"]))
    vals = {}
    for c in wanted:
        best = max((sum(v[c]) / len(v[c]) for v in per_kernel.values() if c in v), default=None)
        if best is not None:
            vals[c] = best
    return vals


def collect_counters(workload: str, fam: Family, params: dict, timeout: int = 180) -> dict:
    """The counter passes of one candidate, each `rocprofv3 --pmc <group> -- python -m ...search --pmc-child`."""
    import glob
    import tempfile
    vals = {}
    root = os.path.dirname(HERE)
    for group in PMC_GROUPS:
        with tempfile.TemporaryDirectory(dir="/tmp") as d:
            cmd = ["rocprofv3", "--pmc", *group, "--output-format", "csv", "-d", d, "-o", "r", "--", sys.executable, "-m",
                   "paper_2602_12305_amd.search", "--workload", workload, "--family", fam.name, "--pmc-child", json.dumps(params)]
            try:
                subprocess.run(cmd, cwd=root, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL, timeout=timeout, check=False,
                               env={**os.environ, "TMPDIR": "/tmp"})
            except (subprocess.TimeoutExpired, OSError):
                continue
            vals.update(main_kernel_counters(glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True), group))
    return vals


class ProfiledEvaluator:
    """evaluate(params) for search(): time and correctness from a worker child (one per search, fed one JSON line per
    candidate), counters from collect_counters() for every correct candidate.  The process that owns this object
    never touches the GPU."""

    def __init__(self, workload: str, fam: Family, steps: int, warmup: int, counters=collect_counters):
        self.workload, self.fam, self.counters = workload, fam, counters
        self.worker = subprocess.Popen([sys.executable, "-m", "paper_2602_12305_amd.search", "--workload", workload, "--family",
                                        fam.name, "--steps", str(steps), "--warmup", str(warmup), "--worker"],
                                       cwd=os.path.dirname(HERE), stdin=subprocess.PIPE, stdout=subprocess.PIPE, text=True)

    def __call__(self, params) -> R.Profile:
        self.worker.stdin.write(json.dumps(params) + "\n")
        self.worker.stdin.flush()
        line = self.worker.stdout.readline()
        while line and not line.startswith("{"):               # anything a library printed on stdout
            line = self.worker.stdout.readline()
        if not line:
            return R.Profile(time=math.inf, correct=False, extra={"why": "worker ended"})
        j = json.loads(line)
        p = R.Profile(time=j["time"] if j["time"] is not None else math.inf, regs=j.get("regs"),
                      scratch_bytes=j.get("scratch_bytes"), correct=j["correct"], extra=j.get("extra", {}))
        if p.correct:
            c = self.counters(self.workload, self.fam, params)
            for k, v in signals(c, p.time).items():
                setattr(p, k, v)
            p.extra["counters"] = c
        return p

    def close(self):
        try:
            self.worker.stdin.close()
            self.worker.wait(timeout=60)
        except Exception:
            self.worker.kill()


def worker_loop(ev: "Evaluator"):
    """Child of ProfiledEvaluator: one candidate per input line, one JSON profile per output line."""
    for line in sys.stdin:
        line = line.strip()
        if not line:
            continue
        p = ev(json.loads(line))
        print(json.dumps({"time": p.time if math.isfinite(p.time) else None, "regs": p.regs, "scratch_bytes": p.scratch_bytes,
                          "correct": bool(p.correct), "extra": p.extra}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="c2_f32_skinny16_silu")
    ap.add_argument("--family", required=True, choices=sorted(FAMILIES))
    ap.add_argument("--budget", type=int, default=24)
    ap.add_argument("--depth", type=int, default=MAX_DEPTH)
    ap.add_argument("--c", type=float, default=UCT_C)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--out", default="")
    ap.add_argument("--layout", type=int, default=-1, help="operand layout for --prebuild (default: the workload's)")
    ap.add_argument("--prebuild", type=int, default=-1,
                    help="only compile every candidate within this many edits of the root (no GPU needed)")
    ap.add_argument("--jobs", type=int, default=8)
    ap.add_argument("--pmc", action="store_true", help="profile every correct candidate with rocprofv3 counter passes")
    ap.add_argument("--worker", action="store_true", help=argparse.SUPPRESS)        # child: time candidates read from stdin
    ap.add_argument("--pmc-child", default="", help=argparse.SUPPRESS)              # child under rocprofv3: launch one candidate
    a = ap.parse_args()
    fam = FAMILIES[a.family]

    if a.worker:
        worker_loop(Evaluator(a.workload, fam, a.steps, a.warmup))
        return
    if a.pmc_child:
        Evaluator(a.workload, fam, 1, 0, with_reference=False).launch_only(json.loads(a.pmc_child))
        return

    if a.prebuild >= 0:
        layout = a.layout if a.layout >= 0 else (1 if a.workload.startswith("c3_") else 0)   # only config 3 has B column-major
        pts = reachable(fam, fam.root, a.prebuild)
        with cf.ThreadPoolExecutor(max_workers=a.jobs) as ex:
            res = list(ex.map(lambda p: build(fam, p, layout), pts))
        print(f"{sum(x is not None for x in res)} of {len(pts)} candidates of {fam.name} built under {CAND}")
        return

    ev = ProfiledEvaluator(a.workload, fam, a.steps, a.warmup) if a.pmc else Evaluator(a.workload, fam, a.steps, a.warmup)
    out = open(a.out, "a") if a.out else None

    def log(n: Node):
        p = n.profile
        rec = {"workload": a.workload, "family": fam.name, "params": n.params, "edit": n.edit, "depth": n.depth,
               "parent": key(n.parent.params) if n.parent else None, "ms": None if not n.alive else round(p.time * 1e3, 5),
               "correct": n.alive, "reward": None if n.reward == -math.inf else round(n.reward, 4), "keep": n.keep,
               "regs": p.regs, "scratch": p.scratch_bytes, **{k: (round(v, 3) if isinstance(v, float) else v)
                                                               for k, v in p.extra.items()}}
        if n.alive and p.sol_sm is not None:
            rec.update({"sol_sm": round(p.sol_sm, 2), "sol_dram": None if p.sol_dram is None else round(p.sol_dram, 2),
                        "dram_bytes": p.dram_bytes, "l1": p.l1, "inst": p.inst, "regime": R.regime(p)})
            if n.parent is not None:
                rec["r_time"] = round(R.time_reward(n.parent.profile.time, p.time), 4)
                rec["r_proxy"] = round(R.proxy_reward(n.parent.profile, p), 4)
                rec["p_guard"] = round(R.guard_penalty(n.parent.profile, p), 4)
        if out:
            out.write(json.dumps(rec) + "\n")
            out.flush()
        ms = f"{p.time * 1e3:9.4f} ms" if n.alive else f"   dead ({p.extra.get('why', 'wrong result')})"
        rw = "   -inf" if n.reward == -math.inf else f"{n.reward:+7.3f}"
        sol = f"  sm {p.sol_sm:5.1f}% dram {p.sol_dram:5.1f}% proxy {rec.get('r_proxy', 0.0):+.3f}" if "sol_sm" in rec and p.sol_dram is not None else ""
        print(f"d{n.depth} {n.edit:16s} {key(n.params):52s} {ms}  R {rw} {'KEEP' if n.keep else '    '}{sol}", flush=True)

    root, nodes = search(fam, fam.root, ev, a.budget, a.depth, a.c, a.seed, log)
    if a.pmc:
        ev.close()
    best, path = best_keep_chain(root)
    print(f"evaluated {len(nodes)} nodes ({len({key(n.params) for n in nodes})} distinct kernels)")
    print("best KEEP chain: " + " -> ".join(f"{key(n.params)} ({n.profile.time * 1e3:.4f} ms)" for n in path))
    print(f"root {root.profile.time * 1e3:.4f} ms, best {best.profile.time * 1e3:.4f} ms, "
          f"speed-up {root.profile.time / best.profile.time:.3f}x")


if __name__ == "__main__":
    main()
