"""The profiler-driven variant sweep (paper section 3.2: every candidate is tested, timed, profiled and scored):
its candidate listing on the host, and a two-variant sweep on the GPU."""
import json
import math
import os
import subprocess
import sys

import pytest

from inputs import synth
from paper_2602_12305_amd import sweep

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_candidate_listing_follows_shape_layout_and_storage_type():
    for name in synth.WORKLOADS + synth.BREADTH_WORKLOADS:
        cands, default_id = sweep.candidates(name)
        names = [n for _, n in cands]
        assert names and "generic_64x64" in names, name
        assert default_id in [i for i, _ in cands], name
        assert name in synth.SPECS and synth.SPECS[name][5] in sweep.PEAK_TFLOPS
    c4 = [n for _, n in sweep.candidates("c4_bf16_8192_silu")[0]]
    assert any(n.startswith("ring_bf16_rr_") for n in c4) and not any("_f32_" in n or "_f16_" in n or "_rc_" in n for n in c4)
    c3 = [n for _, n in sweep.candidates("c3_f32_4096_rc_gelu")[0]]
    assert any(n.startswith("ring_f32_rc_") for n in c3) and not any("_bf16_" in n for n in c3)
    f8 = [n for _, n in sweep.candidates("c4_f8_8192_rc_silu")[0]]
    assert any(n.startswith("ring_f8_rc_") for n in f8)
    # --match narrows, finished (workload, variant) pairs are skipped on a restart
    only, _ = sweep.candidates("c2_f32_skinny16_silu", "skinny_f32")
    assert only and all("skinny_f32" in n for _, n in only)
    rest, _ = sweep.candidates("c2_f32_skinny16_silu", "skinny_f32", done={("c2_f32_skinny16_silu", only[0][1])})
    assert len(rest) == len(only) - 1


@pytest.mark.gpu
def test_two_variant_sweep_scores_against_the_default(tmp_path):
    out = tmp_path / "sweep.jsonl"
    r = subprocess.run([sys.executable, "-m", "paper_2602_12305_amd.sweep", "--workload", "c1_f32_256_relu", "--match", "skinny_f32_wn1_wk4",
                        "--steps", "5", "--warmup", "2", "--pmc", "--out", str(out)], cwd=ROOT, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    recs = [json.loads(line) for line in open(out)]                  # strict JSON: no Infinity
    assert len(recs) >= 2
    for j in recs:
        assert j["correct"] and j["max_err_vs_fallback"] <= 2e-5 and j["ms"] > 0
        assert j["counters"].get("FETCH_SIZE", 0) > 0 and j["counters"].get("SQ_INSTS_VALU", 0) > 0
        assert j["reward_vs_default"] is not None and math.isfinite(j["reward_vs_default"])
    assert "best by reward" in r.stdout
