#!/usr/bin/env python3
"""Benchmark of C = act(A.B + bias) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--all] [--only]

A step is one call of the library on one seeded synthetic workload (inputs resident in HBM
before the timed region; the contraction workloads rotate two buffer sets so that consecutive
steps do not re-read the same bytes from cache).  The headline workload (--workload, default
the memory-bound configuration M=16, N=K=16384, fp32, SiLU) gives `value`; the default run also
times the other four configurations of the benchmark and reports them under "workloads", each
with its own roofline, CPU baseline and parity figure (--only: the headline alone).  --all adds
the breadth workloads (other storage types and layouts on the same shapes) and the siblings:
element-wise ReLU / sigmoid, sum, dot, MSE on 2^28 floats (s_relu, s_sigmoid, s_sum, s_dot,
s_mse), transpose (s_transpose), cross-entropy and LayerNorm (s_ce, s_ln_sample, s_ln_token),
attention (s_mhsa), the contraction fused with the cross-entropy (s_lce, s_lce_f32) and with
LayerNorm (s_gln, s_gln_f32), the block-scaled 4-, 6- and 8-bit contractions (s_mxf4, s_mxf6, s_mxf8; s_mxf4_rows16: 16 rows).
Any of these names can be the headline.  One JSON line is printed.

The "roofline" object prices the dominant kernel of a workload against the published MI355X peak
(HBM 8 TB/s, dense bf16 / fp16 MFMA 2516.6 TFLOP/s, fp8 5033.2, fp6 and fp4 10066.3, fp32 MFMA 157.3) using algorithmic
bytes / flops (one read of the inputs, one write of the outputs; 2*M*N*K flops).  "cpu_baseline" is
the fp64 CPU oracle timed on this host as it stands.  "calibration" holds what the library's two
measuring kernels reach on this board in the same run: the plain copy (HBM) and the register-only
matrix-instruction loop on zeros and on N(0,1) operands (the matrix pipe under the power limit).

Before the W warm-up steps a workload is run back to back for --preheat-ms (300 ms, untimed,
reported as "preheat_ms"): the chip's clocks need some 50 ms of sustained work to reach their
steady values, and 5 warm-up steps of 0.2 ms are over before they have.  For the headline the
figure WITHOUT that pre-heat (W warm-up steps, then K timed ones, on the freshly started process)
is reported as well: "cold_ms_per_step", "cold_value".
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_TFLOPS = {0: 157.3, 1: 2516.6, 2: 2516.6, 3: 5033.2, 4: 10066.3, 5: 5033.2, 6: 10066.3, 7: 10066.3}   # fp32, bf16, fp16, fp8 (E4M3), fp4, fp8 (E5M2), fp6 (E2M3, E3M2) MFMA (dense)
DTYPE_NAME = {0: "f32", 1: "bf16", 2: "f16", 3: "f8e4m3", 4: "f4e2m1", 5: "f8e5m2", 6: "f6e2m3", 7: "f6e3m2"}
# which roof bounds each contraction workload (flop per byte against the ridge of its dtype)
BOUND = {"c1_f32_256_relu": "hbm", "c2_f32_skinny16_silu": "hbm", "c3_f32_4096_rc_gelu": "mfma",
         "c4_bf16_8192_silu": "mfma", "c5_bf16_batched32_relu": "mfma", "c4_f16_8192_silu": "mfma",
         "c2_bf16_skinny16_silu": "hbm", "c4_f8_8192_rc_silu": "mfma", "c4_bf8_8192_rc_silu": "mfma", "c4_f4_8192_rc_silu": "mfma", "c4_f6_8192_rc_silu": "mfma", "c4_bf6_8192_rc_silu": "mfma", "c2_f6_skinny16_rc_silu": "hbm", "c4_bf16_4352_tail_silu": "mfma", "c4_bf16_8192_cr_silu": "mfma",
         "c2_f32_skinny16_rc_silu": "hbm"}
# streaming siblings: (entry point, op, arrays read, arrays written) on 2^28 floats
STREAMS = {"s_relu": ("ew", 0, 1, 1), "s_sigmoid": ("ew", 1, 1, 1), "s_sum": ("red", 0, 1, 0),
           "s_dot": ("red", 1, 2, 0), "s_mse": ("red", 2, 2, 0), "s_transpose": ("tr", 0, 1, 1)}
STREAM_N = 1 << 28
# row-wise siblings: cross-entropy on [8192, 32768] logits; LayerNorm on 64 samples of 64 x 256 x 256
# features (the task's 4-D shape, every feature of a sample is one row) and on 32768 rows of 8192
ROWS = {"s_ce": (8192, 32768), "s_ln_sample": (64, 64 * 256 * 256), "s_ln_token": (32768, 8192)}
# attention: bf16, 4 sequences of 4096 tokens, d_model 2048, 16 heads of 128
MHSA = {"s_mhsa": (4, 4096, 2048, 16)}
# contraction fused with the cross-entropy, B row-major: (M rows, N classes, K, dtype)
LCE = {"s_lce": (8192, 32768, 4096, 1), "s_lce_f32": (4096, 32768, 2048, 0)}
# contraction fused with LayerNorm over each row of the product, B row-major: (M, N, K, dtype)
GLN = {"s_gln": (8192, 8192, 4096, 1), "s_gln_f32": (4096, 4096, 4096, 0)}
# contraction on block-scaled (E8M0 per 32 k) E2M1 or E4M3 operands, k contiguous in both, SiLU: (M, N, K, dtype)
MXF4 = {"s_mxf4": (8192, 8192, 8192, 4), "s_mxf8": (8192, 8192, 8192, 3), "s_mxf6": (8192, 8192, 8192, 6),
        "s_mxf4_rows16": (16, 16384, 16384, 4)}

# HBM bytes per launch of a workload's kernels, from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE
# passes (KiB summed over the kernels of one step, scaled by what the same counters read for the
# library's 1 GiB copy kernel: FETCH_SIZE x 2.0000, WRITE_SIZE x 1.0000; summaries under
# profiles/).  An entry is only reported while the sources of that kernel (its own files and the
# shared epilogue arithmetic) still hash to the value recorded with it.
SKINNY_SRC = ("kernel_skinny.hpp", "kernel_skinny.hip", "kernel_tile_ring.hpp", "epilogue.hpp")
RING_SRC = ("kernel_tile_ring.hpp", "ring_instances.inc", "ring_bf16_rr.hip", "epilogue.hpp")
RINGP_SRC = ("kernel_ring_persistent.hpp",) + RING_SRC
RINGF_SRC = ("kernel_ring_f32.hpp", "ringf_instances.inc", "ring_f32_rc.hip", "kernel_tile_ring.hpp", "epilogue.hpp")
STREAMS_SRC = ("kernel_streams.hip", "epilogue.hpp")
SKINNY16_SRC = ('kernel_skinny16.hpp', 'kernel_skinny16.hip', 'kernel_tile_ring.hpp', 'epilogue.hpp')
LCE_SRC = ('kernel_linear_ce.hip', 'kernel_tile_ring.hpp', 'epilogue.hpp')
LCE_F32_SRC = ('kernel_linear_ce.hip', 'kernel_ring_f32.hpp', 'kernel_tile_ring.hpp', 'epilogue.hpp')
ATTN_SRC = ("kernel_attention.hip", "epilogue.hpp")
TRANSPOSE_SRC = ("kernel_transpose.hip",)
SKINNY_RC_SRC = ("kernel_skinny_rc.hpp", "kernel_skinny_rc.hip", "epilogue.hpp")
RING_F8_SRC = ("kernel_tile_ring.hpp", "ring_instances.inc", "ring_f8_rc.hip", "epilogue.hpp")
RING_BF8_SRC = ("kernel_tile_ring.hpp", "ring_instances.inc", "ring_bf8_rc.hip", "epilogue.hpp")
ROWS_SRC = ("kernel_rows.hip", "epilogue.hpp")
RING_F4_SRC = ("kernel_tile_ring.hpp", "ring_instances.inc", "ring_f4_rc.hip", "epilogue.hpp")
XA_SRC = ("kernel_transpose.hip",) + RING_SRC
GLN_SRC = ("kernel_linear_ln.hip", "kernel_tile_ring.hpp", "epilogue.hpp")
GLN_F32_SRC = ("kernel_linear_ln.hip", "kernel_ring_f32.hpp", "kernel_tile_ring.hpp", "epilogue.hpp")
MX_SRC = ("kernel_mx.hip", "kernel_tile_ring.hpp", "epilogue.hpp")
F6_SRC = ("kernel_f6.hip", "kernel_tile_ring.hpp", "epilogue.hpp")
MX6_SRC = ("kernel_mx.hip", "kernel_f6.hip", "kernel_tile_ring.hpp", "epilogue.hpp")
TRAFFIC = {
    # (workload, kernel variant): per step, all of the step's kernels; KiB figures are FETCH_SIZE and WRITE_SIZE
    ("c1_f32_256_relu", "skinny_f32_dma_wk8_cg1_ns2_nt1"):
        {"bytes": int((827.5 * 2.0 + 256.0) * 1024), "files": SKINNY_SRC, "src": "01c09215cee846dc"},
    ("c2_f32_skinny16_silu", "skinny_f32_dma_wk4_cg2_ns2_nt1"):
        {"bytes": int((531043.4 * 2.0 + 3072.0) * 1024), "files": SKINNY_SRC, "src": "01c09215cee846dc"},
    ("c3_f32_4096_rc_gelu", "ring_f32_rc_128x128_w2x4_ns4"):
        {"bytes": int((385123.2 * 2.0 + 65536.0) * 1024), "files": RINGF_SRC, "src": "f797f1c137a37000"},
    ("c4_bf16_8192_silu", "ring_bf16_rr_256x256_w2x4_ns4_pf"):
        {"bytes": int((798718.6 * 2.0 + 131173.1) * 1024), "files": RING_SRC, "src": "f13a7f529efa5e56"},
    ("c4_f16_8192_silu", "ring_f16_rr_256x256_w2x4_ns4_pf"):
        {"bytes": int((802339.7 * 2.0 + 131101.7) * 1024), "files": RING_SRC, "src": "f13a7f529efa5e56"},
    ("c5_bf16_batched32_relu", "ring_bf16_rr_128x256_w1x4_ns3"):
        {"bytes": int((65939.9 * 2.0 + 262203.0) * 1024), "files": RING_SRC, "src": "f13a7f529efa5e56"},
    ("c2_bf16_skinny16_silu", "skinny_bf16_wn1_wk4_cg2_nt1_split0_il"):
        {"bytes": int((265884.5 * 2.0 + 3584.0) * 1024), "files": SKINNY16_SRC, "src": "90ac2f4cb9357c61"},
    ("c4_f8_8192_rc_silu", "ring_f8_rc_256x256_w2x4_ns5_k64"):
        {"bytes": int((393472.4 * 2.0 + 131087.5) * 1024), "files": RING_F8_SRC, "src": "13396d161ed5b389"},
    ("c4_f4_8192_rc_silu", "ring_f4_rc_256x256_w2x4_ns5_pf"):
        {"bytes": int((196876.6 * 2.0 + 131181.8) * 1024), "files": RING_F4_SRC, "src": "cbc15b94695312f5"},
    ("c4_bf16_8192_cr_silu", "xa_ring"):
        {"bytes": int((863588.1 * 2.0 + 262487.9) * 1024), "files": XA_SRC, "src": "5258360b03c0e65c"},
    ("c2_f32_skinny16_rc_silu", "skinnyrc_f32_dma_wk4_cg4_ns2"):
        {"bytes": int((534585.5 * 2.0 + 1024.0) * 1024), "files": SKINNY_RC_SRC, "src": "49f7af85372c758e"},
    ("s_relu", "s_relu"):
        {"bytes": int((524309.0 * 2.0 + 1048576.8) * 1024), "files": STREAMS_SRC, "src": "a9a12d5504a32b9e"},
    ("s_sigmoid", "s_sigmoid"):
        {"bytes": int((524325.0 * 2.0 + 1048577.4) * 1024), "files": STREAMS_SRC, "src": "a9a12d5504a32b9e"},
    ("s_sum", "s_sum"):
        {"bytes": int((524397.6 * 2.0 + 128.2) * 1024), "files": STREAMS_SRC, "src": "a9a12d5504a32b9e"},
    ("s_dot", "s_dot"):
        {"bytes": int((1048623.7 * 2.0 + 128.3) * 1024), "files": STREAMS_SRC, "src": "a9a12d5504a32b9e"},
    ("s_mse", "s_mse"):
        {"bytes": int((1048626.9 * 2.0 + 128.3) * 1024), "files": STREAMS_SRC, "src": "a9a12d5504a32b9e"},
    ("s_transpose", "s_transpose"):
        {"bytes": int((524321.6 * 2.0 + 1048690.0) * 1024), "files": TRANSPOSE_SRC, "src": "6b1eb4f875ecc63c"},
    ("s_ce", "s_ce"):
        {"bytes": int((525007.2 * 2.0 + 64.1) * 1024), "files": ROWS_SRC, "src": "53d1735df9e83d00"},
    ("s_ln_sample", "s_ln_sample"):
        {"bytes": int((527805.5 * 2.0 + 1053770.3) * 1024), "files": ROWS_SRC, "src": "53d1735df9e83d00"},
    ("s_ln_token", "s_ln_token"):
        {"bytes": int((524319.5 * 2.0 + 1048587.9) * 1024), "files": ROWS_SRC, "src": "53d1735df9e83d00"},
    ("s_mhsa", "mhsa_pingpong_bf16_dk128"):
        {"bytes": int((98427.0 * 2.0 + 65536.0) * 1024), "files": ATTN_SRC, "src": "25b9d901cd9d187e"},
    ("s_lce", "ring_bf16_rr_lse"):
        {"bytes": int((1590397.8 * 2.0 + 33040.0) * 1024), "files": LCE_SRC, "src": "dbb033bc75a3f6a2"},
    ("s_lce_f32", "ring_f32_rr_lse"):
        {"bytes": int((1583694.0 * 2.0 + 32904.0) * 1024), "files": LCE_F32_SRC, "src": "a70c8e7d881d8b06"},
    ("s_gln", "ring_bf16_rr_ln"):
        {"bytes": int((542026.9 * 2.0 + 401408.3) * 1024), "files": GLN_SRC, "src": "11c6767e6b24ac43"},
    ("s_gln_f32", "ring_f32_rr_ln"):
        {"bytes": int((427229.7 * 2.0 + 135282.1) * 1024), "files": GLN_F32_SRC, "src": "071ea73e701ef0ce"},
    ("s_mxf4", "ring_mxf4_rc_256x256_w2x4_ns4_pf"):
        {"bytes": int((211262.8 * 2.0 + 135186.4) * 1024), "files": MX_SRC, "src": "a1d00b0333fcea83"},
    ("c4_bf8_8192_rc_silu", "ring_bf8_rc_256x256_w2x4_ns5_k64"):
        {"bytes": int((393468.5 * 2.0 + 131081.3) * 1024), "files": RING_BF8_SRC, "src": "ea8aadbc474ecf63"},
    ("s_mxf4_rows16", "mx4_dma_cg4_wk3_ns2"):
        {"bytes": int((82943.4 * 2.0 + 512.0) * 1024), "files": MX_SRC, "src": "a1d00b0333fcea83"},
    ("s_mxf8", "ring_mxf8_rc_256x256_w2x4_ns4_k64"):
        {"bytes": int((420185.7 * 2.0 + 139266.2) * 1024), "files": MX_SRC, "src": "a1d00b0333fcea83"},
    ("s_mxf6", "ring_mxf6_rc_256x256_w2x4_ns4_k64"):
        {"bytes": int((469350.6 * 2.0 + 270368.6) * 1024), "files": MX6_SRC, "src": "2a1a93e40738b1aa"},
    ("c4_f6_8192_rc_silu", "xs_ring_f6_rc_256x256_w2x4_ns5_k64"):
        {"bytes": int((442680.1 * 2.0 + 262283.4) * 1024), "files": F6_SRC, "src": "dccd611dbce5e2b7"},
    ("c2_f6_skinny16_rc_silu", "stream6_f6_rc_dma_cg4_wk4_ns2_sub2"):
        {"bytes": int((115496.4 * 2.0 + 512.0) * 1024), "files": F6_SRC, "src": "dccd611dbce5e2b7"},
    ("c4_bf6_8192_rc_silu", "xs_ring_bf6_rc_256x256_w2x4_ns5_k64"):
        {"bytes": int((442671.7 * 2.0 + 262225.2) * 1024), "files": F6_SRC, "src": "dccd611dbce5e2b7"},
}


def kernel_source_hash(files):
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2602_12305_amd", "csrc")
    for f in files:
        h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:16]


def traffic_of(workload, kernel):
    tr = TRAFFIC.get((workload, kernel))
    if not tr:
        return None
    return tr["bytes"] if tr["src"] == kernel_source_hash(tr["files"]) else None


class Case:
    """One workload set up on the GPU: `step(i)` enqueues one pass; `bound`, `flops`, `nbytes` (algorithmic),
    `dtype` (code), `kernel` (the dominant kernel's name) and `config` describe it; `check()` times the oracle on
    a bounded sample and returns (cpu_baseline object, parity key, parity value)."""
    name = kernel = ""
    bound = "hbm"
    flops = nbytes = 0.0
    dtype = 0
    config = {}

    def step(self, i):
        raise NotImplementedError

    def check(self):
        raise NotImplementedError

    def roof_value(self, ms):
        return self.nbytes / (ms * 1e-3) / 1e9 if self.bound == "hbm" else self.flops / (ms * 1e-3) / 1e12

    @property
    def peak(self):
        return PEAK_HBM_GBS if self.bound == "hbm" else PEAK_TFLOPS[self.dtype]

    @property
    def unit(self):
        return "GB/s" if self.bound == "hbm" else "TFLOP/s"

    def baseline(self, oracle, secs, fraction, sample):
        """cpu_baseline object: the oracle took `secs` for `fraction` of the workload."""
        full = secs / fraction
        val = (self.nbytes / 1e9 if self.bound == "hbm" else self.flops / 1e12) / full
        return {"value": float(f"{val:.4g}"), "unit": self.unit, "cores": oracle.num_threads(), "kind": "oracle",
                "sample": sample, "seconds": round(secs, 3)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--preheat-ms", type=float, default=300.0,
                    help="run the workload back to back for this long before the warm-up steps (clocks at steady state)")
    ap.add_argument("--workload", default="c2_f32_skinny16_silu")
    ap.add_argument("--all", action="store_true", help="also time the breadth workloads and the siblings")
    ap.add_argument("--only", action="store_true", help="time the headline workload alone (no other configurations)")
    ap.add_argument("--variant", type=int, default=-1, help="force one kernel variant for the headline (default: dispatcher)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-gib", type=float, default=0.0,
                    help="instead of a workload, time the library's plain copy kernel on this many GiB "
                         "(HBM ceiling and calibration of the profiler's byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this library runs on one GPU; there is no multi-GPU path to time (use --gpus 1)",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from inputs import synth
    from paper_2602_12305_amd import binding as ob

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    def to_dev(x):
        return torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x).cuda()

    def run_timed(step, steps, warmup, preheat_ms):
        """`preheat_ms` of untimed back-to-back calls (the chip's clocks take some 50 ms of sustained work to reach
        their steady values: the headline workload after 5 warm-up steps 0.194 ms per step, after 85 ms of the
        same work 0.170 ms, on one board, alternating), W warm-up steps, then exactly K timed steps between two
        synchronisations.  Returns (whole-step ms by the host clock or the device's, whichever is longer; ms by
        HIP events on the launch stream)."""
        if preheat_ms > 0:
            t_end = time.perf_counter() + preheat_ms * 1e-3
            i = 0
            while time.perf_counter() < t_end:
                for _ in range(16):
                    step(i)
                    i += 1
                torch.cuda.synchronize()
        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for i in range(steps):
            step(i)
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        dev_ms = e0.elapsed_time(e1)
        return max(wall_ms, dev_ms) / steps, dev_ms / steps

    def measure(case, with_oracle, cold=False):
        """Time one case; the result object every workload shares."""
        res = {"workload": case.name, "variant": case.kernel, "dtype": DTYPE_NAME[case.dtype]}
        if cold:
            cms, ckms = run_timed(case.step, args.steps, args.warmup, 0.0)
            res["cold_ms_per_step"] = round(cms, 5)
            res["cold_value"] = round(case.roof_value(cms), 3)
            res["cold_frac"] = round(case.roof_value(ckms) / case.peak, 4)
        ms, kernel_ms = run_timed(case.step, args.steps, args.warmup, args.preheat_ms)
        achieved = case.roof_value(kernel_ms)
        res.update({"ms_per_step": round(ms, 5), "value": round(case.roof_value(ms), 3), "unit": case.unit,
                    "GB/s": round(case.nbytes / (ms * 1e-3) / 1e9, 2),
                    "hbm_frac": round(case.nbytes / (kernel_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)})
        if case.flops:
            res["TFLOP/s"] = round(case.flops / (ms * 1e-3) / 1e12, 3)
            res["mfma_frac"] = round(case.flops / (kernel_ms * 1e-3) / 1e12 / PEAK_TFLOPS[case.dtype], 4)
        res["roofline"] = {"bound": case.bound, "achieved": round(achieved, 3), "peak": case.peak, "unit": case.unit,
                           "frac": round(achieved / case.peak, 4), "traffic": traffic_of(case.name, case.kernel),
                           "kernel": case.kernel, "kernel_ms": round(kernel_ms, 5)}
        res["config"] = dict(case.config, workload=case.name)
        if with_oracle:
            base, key, err = case.check()
            res["cpu_baseline"] = base
            res[key] = float(f"{err:.3e}")
        return res

    # ---- the cases -------------------------------------------------------------------------------------------

    class Gemm(Case):
        """C = act(A.B + bias) on one of the benchmark's configurations or breadth workloads."""

        def __init__(self, name, variant=-1):
            w = self.w = synth.make_workload(name)
            self.name, self.bound, self.dtype = name, BOUND[name], w.dtype
            self.flops, self.nbytes = float(w.flops), float(w.algorithmic_bytes)
            num, den = (2, 1) if w.dtype == 4 else (4, 3) if w.dtype in (6, 7) else (1, 1)     # E2M1: two elements a byte; 6-bit: four in three
            self.lda, self.ldb = w.A.shape[-1] * num // den, w.B.shape[-1] * num // den
            self.sA = w.A.shape[-2] * self.lda if w.batch > 1 else 0
            self.sB = w.B.shape[-2] * self.ldb if w.batch > 1 else 0
            self.sBias = w.N if w.batch > 1 else 0
            self.sets = []
            for _ in range(2):
                Cd = torch.empty((w.batch, w.M, w.N), dtype=torch.float32 if w.dtype == 0 else torch.int16, device="cuda")
                self.sets.append((to_dev(w.A), to_dev(w.B), to_dev(w.bias), Cd))
            s = self.sets[0]
            probe = (w.batch, w.M, w.N, w.K, s[0], self.lda, self.sA, s[1], self.ldb, self.sB, s[2], self.sBias,
                     s[3], w.N, w.M * w.N, w.layout, w.dtype, w.act)
            self.vid = variant if variant >= 0 else ob.optiml_select_variant(*probe)
            self.kernel = ob.optiml_variant_name(self.vid)
            self.config = {"batch": w.batch, "M": w.M, "N": w.N, "K": w.K, "layout": ["rr", "rc", "cr", "cc"][w.layout],
                           "act": ["none", "relu", "gelu_tanh", "silu"][w.act], "variant": self.kernel}
            self.last = 0

        def step(self, i):
            w = self.w
            Ad, Bd, bd, Cd = self.sets[i & 1]
            self.last = i & 1
            ob.optiml_gemm_epilogue_variant(w.batch, w.M, w.N, w.K, Ad, self.lda, self.sA, Bd, self.ldb, self.sB, bd,
                                            self.sBias, Cd, w.N, w.M * w.N, w.layout, w.dtype, w.act, self.vid)

        def check(self):
            import oracle
            w = self.w
            # bounded sample of the same workload: the whole output up to 8e10 multiply-adds, else seeded sampled entries
            t0 = time.perf_counter()
            if w.flops // 2 <= 8e10:
                ref = oracle.gemm_epilogue(w.A, w.B, w.bias, w.M, w.N, w.K, dtype=w.dtype, act=w.act, layout=w.layout,
                                           batch=w.batch)
                secs = time.perf_counter() - t0
                frac, sample, idx = 1.0, "whole workload", None
            else:
                idx = synth.sample_entries(w.seed, 1 << 20, w.batch, w.M, w.N)
                ref = oracle.gemm_epilogue_sampled(*idx, w.A, w.B, w.bias, w.M, w.N, w.K, dtype=w.dtype, act=w.act,
                                                   layout=w.layout, batch=w.batch)
                secs = time.perf_counter() - t0
                frac = len(idx[0]) / float(w.batch * w.M * w.N)
                sample = f"{len(idx[0])} sampled output entries of {w.batch * w.M * w.N}"
            got = self.sets[self.last][3].cpu().numpy()
            if w.dtype != 0:
                got = synth.from_bits(got.view(np.uint16), 1 if w.dtype >= 3 else w.dtype)      # 8-, 6- and 4-bit operands: bf16 result
            got = got.astype(np.float64)
            if idx is not None:
                got = got[idx]
            rho = float(np.sqrt(np.mean(ref * ref)))
            e1 = float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rho)))
            return self.baseline(oracle, secs, frac, sample), "parity_e1", e1

    class Stream(Case):
        """One streaming sibling on 2^28 seeded uniform floats (1 GiB per array)."""

        def __init__(self, name):
            self.name = self.kernel = name
            self.kind, self.op, reads, writes = STREAMS[name]
            n = self.n = STREAM_N
            gen = lambda tag: synth.uniform(7, tag, n >> 16, 1 << 16, -2.0, 2.0).reshape(-1)
            self.hx = gen("x")
            self.hy = gen("y") if reads == 2 else None
            self.xd = torch.from_numpy(self.hx).cuda()
            self.yd = torch.from_numpy(self.hy).cuda() if self.hy is not None else None
            self.od = torch.empty(1 if self.kind == "red" else n, dtype=torch.float32, device="cuda")
            self.side = 1 << 14                                     # the transpose sees the array as 16384 x 16384
            self.nbytes = float(4 * n * (reads + writes) + (4 if self.kind == "red" else 0))
            self.config = {"n": n}

        def step(self, i):
            if self.kind == "ew":
                ob.optiml_elementwise(self.n, self.xd, self.od, self.op)
            elif self.kind == "tr":
                ob.optiml_transpose(self.side, self.side, self.xd, self.side, self.od, self.side, 4)
            else:
                ob.optiml_reduce(self.n, self.xd, self.yd, self.op, self.od)

        def check(self):
            import oracle
            n = self.n
            t0 = time.perf_counter()
            if self.kind == "ew":
                m = 1 << 24                                         # bounded sample: the first 2^24 elements
                ref = oracle.elementwise(self.hx[:m], self.op)
                secs = time.perf_counter() - t0
                got = self.od[:m].cpu().numpy().astype(np.float64)
                err = float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-30)))
                return self.baseline(oracle, secs, m / n, f"first {m} of {n} elements"), "parity_rel_err", err
            if self.kind == "tr":
                ref = oracle.transpose(self.hx.reshape(self.side, self.side))
                secs = time.perf_counter() - t0
                err = 0.0 if np.array_equal(self.od.cpu().numpy().reshape(self.side, self.side), ref) else 1.0
            else:
                ref = oracle.reduce(self.hx, self.hy, self.op)
                secs = time.perf_counter() - t0
                err = abs(float(self.od.item()) - ref) / max(abs(ref), 1e-30)
            return self.baseline(oracle, secs, 1.0, "whole workload"), "parity_rel_err", err

    class Rows(Case):
        """Cross-entropy or LayerNorm on a seeded normal array of 1 GiB."""

        def __init__(self, name):
            self.name = self.kernel = name
            rows, cols = self.rows, self.cols = ROWS[name]
            self.hx = synth.normal(8, "x", rows, cols, 0.5, 2.0)
            self.xd = torch.from_numpy(self.hx).cuda()
            if name == "s_ce":
                self.hl = (np.arange(rows, dtype=np.int64) * 7919 % cols).astype(np.int32)
                self.ld = torch.from_numpy(self.hl).cuda()
                self.od = torch.empty(1, dtype=torch.float32, device="cuda")
                self.nbytes = float(4 * rows * cols + 4 * rows + 4)
            else:
                self.od = torch.empty_like(self.xd)
                self.nbytes = float(8 * rows * cols)
            self.config = {"rows": rows, "cols": cols, "n": rows * cols}

        def step(self, i):
            if self.name == "s_ce":
                ob.optiml_cross_entropy(self.rows, self.cols, self.xd, self.cols, self.ld, self.od)
            else:
                ob.optiml_layernorm(self.rows, self.cols, self.xd, self.od, 1e-5)

        def check(self):
            import oracle
            t0 = time.perf_counter()
            if self.name == "s_ce":
                ref = oracle.cross_entropy(self.hx, self.hl)
                secs = time.perf_counter() - t0
                return self.baseline(oracle, secs, 1.0, "whole workload"), "parity_abs_err", abs(float(self.od.item()) - ref)
            m = max(1, self.rows // 16)                             # bounded sample: the first sixteenth of the rows
            ref = oracle.layernorm(self.hx[:m], 1e-5)
            secs = time.perf_counter() - t0
            err = float(np.max(np.abs(self.od[:m].cpu().numpy().astype(np.float64) - ref)))
            return self.baseline(oracle, secs, m / self.rows, f"first {m} of {self.rows} rows"), "parity_abs_err", err

    class Mhsa(Case):
        """Multi-head self-attention, bf16 storage, seeded N(0, 1) inputs."""
        bound, dtype, kernel = "mfma", 1, "mhsa_pingpong_bf16_dk128"

        def __init__(self, name):
            self.name = name
            batch, N, d, heads = self.shape = MHSA[name]
            self.host = [synth.f32_to_bf16_bits(synth.normal(9, tag, N, d, batch=batch)) for tag in ("q", "k", "v")]
            self.Qd, self.Kd, self.Vd = (torch.from_numpy(h.view(np.int16)).cuda() for h in self.host)
            self.Od = torch.empty_like(self.Qd)
            self.flops = 4.0 * batch * N * N * d                    # two products of 2 N^2 d_k flops per head
            self.nbytes = 4.0 * batch * N * d * 2
            self.config = {"batch": batch, "N": N, "d_model": d, "heads": heads}

        def step(self, i):
            batch, N, d, heads = self.shape
            ob.optiml_mhsa(batch, N, d, heads, self.Qd, self.Kd, self.Vd, self.Od, 1)

        def check(self):
            import oracle
            batch, N, d, heads = self.shape
            t0 = time.perf_counter()
            ref = oracle.mhsa(self.host[0][:1], self.host[1][:1], self.host[2][:1], heads, dtype=oracle.BF16)[0]
            secs = time.perf_counter() - t0
            got = synth.bf16_bits_to_f32(self.Od[0].cpu().numpy().view(np.uint16)).astype(np.float64)
            rho = float(np.sqrt(np.mean(ref * ref)))
            err = float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rho)))
            return self.baseline(oracle, secs, 1.0 / batch, f"sequence 0 of {batch} (all {heads} heads)"), "parity_e1", err

    class Lce(Case):
        """Contraction + cross-entropy: A N(0, 1/K) (logits of unit variance), B N(0,1), bias N(0,1)."""
        bound = "mfma"

        def __init__(self, name):
            self.name = name
            M, N, K, dt = self.shape = LCE[name]
            self.dtype = dt
            self.kernel = f"ring_{DTYPE_NAME[dt]}_rr_lse"
            self.A = synth.to_bits(synth.normal(10, "A", M, K, 0.0, K ** -0.5), dt)
            self.B = synth.to_bits(synth.normal(10, "B", K, N), dt)
            self.bias = synth.normal(10, "bias", 1, N)[0]
            self.labels = ((7919 * np.arange(M)) % N).astype(np.int32)
            self.Ad, self.Bd = (torch.from_numpy(h.view(np.int16) if dt else h).cuda() for h in (self.A, self.B))
            self.bd, self.ld = torch.from_numpy(self.bias).cuda(), torch.from_numpy(self.labels).cuda()
            self.out = torch.empty(2, dtype=torch.float32, device="cuda")
            assert ob.optiml_gemm_cross_entropy_path(M, N, K, self.Ad, K, self.Bd, N, self.bd, 0, dt) == 0
            self.flops = 2.0 * M * N * K
            self.nbytes = float((M * K + K * N) * (2 if dt else 4) + 4 * N + 4 * M + 4)
            self.config = {"M": M, "N": N, "K": K}

        def step(self, i, rows=None, o=0):
            M, N, K, dt = self.shape
            ob.optiml_gemm_cross_entropy(rows or M, N, K, self.Ad, K, self.Bd, N, self.bd, self.ld, self.out[o:], 0, dt)

        def check(self):
            import oracle
            M, N, K, dt = self.shape
            m = M // 2                                              # bounded sample: the first half of the rows
            self.step(0, m, 1)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ref = oracle.gemm_cross_entropy(self.A[:m], self.B, self.bias, self.labels[:m], m, N, K, dtype=dt)
            secs = time.perf_counter() - t0
            return (self.baseline(oracle, secs, m / M, f"first {m} of {M} rows"), "parity_abs_err",
                    abs(float(self.out[1].item()) - ref))

    class Gln(Case):
        """Contraction + LayerNorm over the rows of the product: A N(0, 1/K), B N(0,1), bias N(1.5, 3^2)."""
        bound = "mfma"

        def __init__(self, name):
            self.name = name
            M, N, K, dt = self.shape = GLN[name]
            self.dtype = dt
            self.kernel = f"ring_{DTYPE_NAME[dt]}_rr_ln"
            self.A = synth.to_bits(synth.normal(13, "A", M, K, 0.0, K ** -0.5), dt)
            self.B = synth.to_bits(synth.normal(13, "B", K, N), dt)
            self.bias = synth.normal(13, "bias", 1, N, 1.5, 3.0)[0]
            self.Ad, self.Bd = (torch.from_numpy(h.view(np.int16) if dt else h).cuda() for h in (self.A, self.B))
            self.bd = torch.from_numpy(self.bias).cuda()
            self.Y = torch.empty((M, N), dtype=torch.int16 if dt else torch.float32, device="cuda")
            assert ob.optiml_gemm_layernorm_path(M, N, K, self.Ad, K, self.Bd, N, self.bd, self.Y, N, 0, dt) == 0
            self.flops = 2.0 * M * N * K
            self.nbytes = float((M * K + K * N + M * N) * (2 if dt else 4) + 4 * N)
            self.config = {"M": M, "N": N, "K": K}

        def step(self, i):
            M, N, K, dt = self.shape
            ob.optiml_gemm_layernorm(M, N, K, self.Ad, K, self.Bd, N, self.bd, self.Y, N, 1e-5, 0, dt)

        def check(self):
            import oracle
            M, N, K, dt = self.shape
            m = 256                                                 # bounded sample: the first 256 rows, whole rows
            t0 = time.perf_counter()
            ref = oracle.gemm_layernorm(self.A[:m], self.B, self.bias, m, N, K, dtype=dt, eps=1e-5)
            secs = time.perf_counter() - t0
            got = self.Y[:m].cpu().numpy()
            got = (synth.from_bits(got.view(np.uint16), dt) if dt else got).astype(np.float64)
            return (self.baseline(oracle, secs, m / M, f"first {m} of {M} rows"), "parity_abs_err",
                    float(np.max(np.abs(got - ref))))

    class Mx(Case):
        """Block-scaled E2M1, E2M3 or E4M3 contraction: N(0, 1) operands whose 32-blocks vary in magnitude over 2^+-3, quantised
        block by block (scale = the block's largest magnitude brought into the element type's range), bias N(0, 1), SiLU."""
        bound = "mfma"

        def __init__(self, name):
            M, N, K, self.dtype = MXF4[name]
            self.shape = (M, N, K)
            self.name = name
            self.kernel = {4: "ring_mxf4_rc_256x256_w2x4_ns4_pf", 6: "ring_mxf6_rc_256x256_w2x4_ns4_k64"}.get(self.dtype, "ring_mxf8_rc_256x256_w2x4_ns4_k64")
            if M <= 128:
                self.kernel, self.bound = "mx4_dma_cg4_wk3_ns2", "hbm"
            bits = {4: 4, 6: 6}.get(self.dtype, 8)            # per stored element
            def operand(tag, rows):
                x = synth.normal(17, tag, rows, K)
                e = synth.integers(18, tag + "e", rows, K // 32, -3, 3)
                return synth.mx_quantize(x * np.repeat(np.exp2(e), 32, axis=1).astype(np.float32), self.dtype)
            (self.A, self.sA), (self.B, self.sB) = operand("A", M), operand("B", N)
            self.bias = synth.normal(17, "bias", 1, N)[0]
            self.dev = [torch.from_numpy(np.ascontiguousarray(h)).cuda() for h in (self.A, self.sA, self.B, self.sB, self.bias)]
            self.C = torch.empty((M, N), dtype=torch.int16, device="cuda")
            Ad, sAd, Bd, sBd, bd = self.dev
            assert ob.optiml_gemm_epilogue_mx_path(M, N, K, Ad, K, sAd, K // 32, Bd, K, sBd, K // 32, bd, self.C, N, self.dtype) == (2 if M <= 128 else 0)
            self.flops = 2.0 * M * N * K
            self.nbytes = float((M + N) * (K * bits // 8 + K // 32) + 2 * M * N + 4 * N)
            self.config = {"M": M, "N": N, "K": K, "layout": "rc", "act": "silu", "block": 32}

        def step(self, i):
            M, N, K = self.shape
            Ad, sAd, Bd, sBd, bd = self.dev
            ob.optiml_gemm_epilogue_mx(M, N, K, Ad, K, sAd, K // 32, Bd, K, sBd, K // 32, bd, self.C, N, self.dtype, 3)

        def check(self):
            import oracle
            M, N, K = self.shape
            rows = np.arange(0, M, max(1, M // 512))[:512]; cols = np.arange(0, N, N // 1024)[:1024] + 1    # bounded sample: 512 x 1024 entries
            t0 = time.perf_counter()
            take = lambda a, i: np.ascontiguousarray(a[i])
            ref = oracle.gemm_epilogue_mx(take(self.A, rows), take(self.sA, rows), take(self.B, cols), take(self.sB, cols),
                                          self.bias[cols], len(rows), len(cols), K, dtype=self.dtype, act=3)
            secs = time.perf_counter() - t0
            got = synth.bf16_bits_to_f32(self.C.cpu().numpy().view(np.uint16)[np.ix_(rows, cols)]).astype(np.float64)
            rho = float(np.sqrt(np.mean(ref * ref)))
            e1 = float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rho)))
            return (self.baseline(oracle, secs, ref.size / float(M * N), f"{ref.size} entries of {M * N} (512 rows x 1024 columns)"),
                    "parity_e1", e1)

    def make_case(name, variant=-1):
        if name in BOUND:
            return Gemm(name, variant)
        for table, cls in ((STREAMS, Stream), (ROWS, Rows), (MHSA, Mhsa), (LCE, Lce), (GLN, Gln), (MXF4, Mx)):
            if name in table:
                return cls(name)
        raise SystemExit(f"bench.py: unknown workload {name}")

    # ---- calibration: what the library's two measuring kernels reach on this board ------------------------------

    def calibrate():
        out = {}
        nbytes = 1 << 30
        src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        ms, _ = run_timed(lambda i: ob.optiml_copy_bytes(dst, src, nbytes), 20, 3, 100.0)
        out["copy_GBs"] = round(2 * nbytes / (ms * 1e-3) / 1e9, 1)
        del src, dst
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        n16 = cus * 32768                                           # 16-bit operand values the probe may read
        sink = torch.empty(cus * 256, dtype=torch.float32, device="cuda")
        normal = synth.f32_to_bf16_bits(synth.normal(12, "probe", n16 >> 10, 1 << 10)).view(np.int16).reshape(-1)
        for tag, host, reads in (("zeros", np.zeros(n16, dtype=np.int16), 0), ("normal", normal, 0),
                                 ("normal_lds8", normal, 8), ("normal_lds12", normal, 12)):
            ops = torch.from_numpy(host).cuda()
            flops = [0.0]

            def probe(i):
                flops[0] = ob.optiml_mfma_probe(ops, n16 * 2, sink, cus * 256, 4000, 1, reads)
            ms, _ = run_timed(probe, 20, 3, 300.0)
            out[f"mfma_bf16_{tag}_TFLOPs"] = round(flops[0] / (ms * 1e-3) / 1e12, 1)
        out["note"] = ("plain 1 GiB copy (read + write); loop of 32x32x16 bf16 matrix instructions with no global-memory "
                       "traffic on all-zero and on N(0,1) operands held in registers, and on N(0,1) operands read from "
                       "LDS at 8 or 12 fragment reads per 16 instructions (128x128 / 128x64 wave tiles): the board's "
                       "own ceilings under its power limit")
        return out

    if args.copy_gib > 0:
        nbytes = int(args.copy_gib * (1 << 30)) // 16 * 16
        src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        ms, _ = run_timed(lambda i: ob.optiml_copy_bytes(dst, src, nbytes), args.steps, args.warmup, 0.0)
        print(json.dumps({"metric": "GB/s of a plain device copy (bytes read + bytes written)", "unit": "GB/s",
                          "value": round(2 * nbytes / (ms * 1e-3) / 1e9, 1), "bytes_read": nbytes,
                          "bytes_written": nbytes, "ms_per_step": round(ms, 5), "steps": args.steps,
                          "frac_of_8TBs": round(2 * nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}))
        return

    # ---- the run ---------------------------------------------------------------------------------------------

    with_oracle = not args.no_cpu_baseline
    case = make_case(args.workload, args.variant)
    head = measure(case, with_oracle, cold=True)
    del case
    torch.cuda.empty_cache()
    what = {"hbm": "GB/s (algorithmic bytes) of ", "mfma": "TFLOP/s of "}[head["roofline"]["bound"]]
    label = "act(A.B+bias)" if args.workload in BOUND else args.workload[2:]
    out = {"metric": what + label, "value": head["value"], "unit": head["unit"], "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "preheat_ms": args.preheat_ms, "ms_per_step": head["ms_per_step"],
           "cold_ms_per_step": head["cold_ms_per_step"], "cold_value": head["cold_value"],
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"],
           "data": "synthetic", "config": head["config"], "roofline": head["roofline"]}
    for k in ("TFLOP/s", "GB/s", "cpu_baseline", "parity_e1", "parity_rel_err", "parity_abs_err"):
        if k in head:
            out[k] = head[k]

    others = []
    if not args.only:
        others += [n for n in synth.WORKLOADS if n != args.workload]
    if args.all:
        others += [n for n in list(synth.BREADTH_WORKLOADS) + list(STREAMS) + list(ROWS) + list(MHSA) + list(LCE) + list(GLN) + list(MXF4)
                   if n != args.workload and n not in others]
    if others:
        out["workloads"] = {args.workload: head}
        for name in others:
            c = make_case(name)
            # the oracle beside every configuration of the benchmark; the breadth workloads and siblings are timed only
            out["workloads"][name] = measure(c, with_oracle and name in synth.WORKLOADS)
            del c
            torch.cuda.empty_cache()
    if not args.only:
        out["calibration"] = calibrate()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
