#!/usr/bin/env python3
"""Benchmark of C = act(A.B + bias) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--all]

A step is one call of the library on one seeded synthetic workload (inputs resident in
HBM before the timed region; two rotating buffer sets so that consecutive steps do not
re-read the same bytes from cache).  The default workload is the memory-bound skinny
configuration (M=16, N=K=16384, fp32, SiLU); --all also times the other four and the
streaming siblings (element-wise ReLU / sigmoid, sum, dot, MSE on 2^28 floats: --workload
s_relu, s_sigmoid, s_sum, s_dot, s_mse; cross-entropy and LayerNorm: s_ce, s_ln_sample,
s_ln_token; transpose: s_transpose; attention: s_mhsa; contraction + cross-entropy: s_lce) and adds them under "workloads".  One JSON line is
printed.

The "roofline" object prices the dominant kernel of the workload against the published
MI355X peak (HBM 8 TB/s, dense bf16 MFMA 2516.6 TFLOP/s, fp32 MFMA 157.3 TFLOP/s) using
algorithmic bytes / flops (one read of A, B, bias, one write of C; 2*M*N*K flops).
"cpu_baseline" is the fp64 CPU oracle timed on this host as it stands.

Before the W warm-up steps the workload is run back to back for --preheat-ms (300 ms, untimed,
reported as "preheat_ms"): the chip's clocks need some 50 ms of sustained work to reach their
steady values, and 5 warm-up steps of 0.2 ms are over before they have.
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
PEAK_TFLOPS = {0: 157.3, 1: 2516.6, 2: 2516.6, 3: 5033.2}          # fp32, bf16, fp16, fp8 MFMA (dense)
# which roof bounds each workload (flop per byte against the ridge of its dtype)
BOUND = {"c1_f32_256_relu": "hbm", "c2_f32_skinny16_silu": "hbm", "c3_f32_4096_rc_gelu": "mfma",
         "c4_bf16_8192_silu": "mfma", "c5_bf16_batched32_relu": "mfma", "c4_f16_8192_silu": "mfma", "c2_bf16_skinny16_silu": "hbm", "c4_f8_8192_rc_silu": "mfma", "c4_bf16_8192_cr_silu": "mfma", "c2_f32_skinny16_rc_silu": "hbm"}
DTYPE_NAME = {0: "f32", 1: "bf16", 2: "f16", 3: "f8e4m3"}
# streaming siblings: (entry point, op, arrays read, arrays written)
STREAMS = {"s_relu": ("ew", 0, 1, 1), "s_sigmoid": ("ew", 1, 1, 1), "s_sum": ("red", 0, 1, 0),
           "s_dot": ("red", 1, 2, 0), "s_mse": ("red", 2, 2, 0), "s_transpose": ("tr", 0, 1, 1)}
STREAM_N = 1 << 28
# row-wise siblings: cross-entropy on [8192, 32768] logits; LayerNorm on 64 samples of 64 x 256 x 256
# features (the task's 4-D shape, every feature of a sample is one row) and on 32768 rows of 8192
# attention: bf16, 4 sequences of 4096 tokens, d_model 2048, 16 heads of 128
MHSA = {"s_mhsa": (4, 4096, 2048, 16)}
# contraction fused with the cross-entropy, B row-major: 8192 rows (tokens), 32768 classes, K 4096 in bf16;
# 4096 rows, 32768 classes, K 2048 in fp32
LCE = {"s_lce": (8192, 32768, 4096, 1), "s_lce_f32": (4096, 32768, 2048, 0)}     # (M, N, K, dtype)
ROWS = {"s_ce": (8192, 32768), "s_ln_sample": (64, 64 * 256 * 256), "s_ln_token": (32768, 8192)}

# HBM bytes per launch of a workload's kernels, from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE
# passes (KiB summed over the kernels of one step, scaled by what the same counters read for the library's 1 GiB copy
# kernel: FETCH_SIZE x 2.0000, WRITE_SIZE x 1.0000; summaries under profiles/).  An entry is only
# reported while the sources of that kernel (its own files and the shared epilogue arithmetic) still hash to
# the value recorded with it.
SKINNY_SRC = ("kernel_skinny.hpp", "kernel_skinny.hip", "epilogue.hpp")
RING_SRC = ("kernel_tile_ring.hpp", "ring_instances.inc", "ring_bf16_rr.hip", "epilogue.hpp")
RINGP_SRC = ("kernel_ring_persistent.hpp",) + RING_SRC
RINGF_SRC = ("kernel_ring_f32.hpp", "ringf_instances.inc", "ring_f32_rc.hip", "kernel_tile_ring.hpp", "epilogue.hpp")
STREAMS_SRC = ("kernel_streams.hip", "epilogue.hpp")
SKINNY16_SRC = ('kernel_skinny16.hpp', 'kernel_skinny16.hip', 'epilogue.hpp')
LCE_SRC = ('kernel_linear_ce.hip', 'kernel_tile_ring.hpp', 'epilogue.hpp')
LCE_F32_SRC = ('kernel_linear_ce.hip', 'kernel_ring_f32.hpp', 'kernel_tile_ring.hpp', 'epilogue.hpp')
ATTN_SRC = ("kernel_attention.hip", "epilogue.hpp")
TRANSPOSE_SRC = ("kernel_transpose.hip",)
SKINNY_RC_SRC = ("kernel_skinny_rc.hpp", "kernel_skinny_rc.hip", "epilogue.hpp")
RING_F8_SRC = ("kernel_tile_ring.hpp", "ring_instances.inc", "ring_f8_rc.hip", "epilogue.hpp")
ROWS_SRC = ("kernel_rows.hip", "epilogue.hpp")
TRAFFIC = {
    # (workload, kernel variant): per step, all of the step's kernels; KiB figures are FETCH_SIZE and WRITE_SIZE
    ("c2_f32_skinny16_silu", "skinny_f32_wn1_wk8_cg2_nt1_split0_il"):
        {"bytes": int((529551.0 * 2.0 + 3072.0) * 1024), "files": SKINNY_SRC, "src": "d4ff8d1267cf9162"},
    ("c3_f32_4096_rc_gelu", "ring_f32_rc_128x128_w2x4_ns4"):
        {"bytes": int((385145.3 * 2.0 + 65536.0) * 1024), "files": RINGF_SRC, "src": "3d144bf02577476c"},
    ("c4_bf16_8192_silu", "ring_bf16_rr_256x256_w2x4_ns4_pf"):
        {"bytes": int((806644.5 * 2.0 + 131072.1) * 1024), "files": RING_SRC, "src": "7a5f3f964118548f"},
    ("c4_f16_8192_silu", "ring_f16_rr_256x256_w2x4_ns4_pf"):
        {"bytes": int((813173.6 * 2.0 + 131072.0) * 1024), "files": RING_SRC, "src": "7a5f3f964118548f"},
    ("c5_bf16_batched32_relu", "ringp_bf16_rr_256x256_w2x4_ns4"):
        {"bytes": int((69975.3 * 2.0 + 266658.2) * 1024), "files": RINGP_SRC, "src": "b23f7957bb0ba2b5"},
    ("c2_bf16_skinny16_silu", "skinny_bf16_wn1_wk4_cg2_nt1_split0_il"):
        {"bytes": int((266407.9 * 2.0 + 4608.0) * 1024), "files": SKINNY16_SRC, "src": "52329cc04db85d01"},
    ("s_sigmoid", "s_sigmoid"):
        {"bytes": int((524327.4 * 2.0 + 1048576.7) * 1024), "files": STREAMS_SRC, "src": "e21a390bc9b59339"},
    ("s_dot", "s_dot"):
        {"bytes": int((1048631.8 * 2.0 + 128.3) * 1024), "files": STREAMS_SRC, "src": "e21a390bc9b59339"},
    ("s_ce", "s_ce"):
        {"bytes": int((524988.0 * 2.0 + 64.1) * 1024), "files": ROWS_SRC, "src": "cf001e03e5c57dd6"},
    ("s_ln_sample", "s_ln_sample"):
        {"bytes": int((1049946.3 * 2.0 + 1049990.3) * 1024), "files": ROWS_SRC, "src": "cf001e03e5c57dd6"},
    ("s_ln_token", "s_ln_token"):
        {"bytes": int((524321.3 * 2.0 + 1048587.4) * 1024), "files": ROWS_SRC, "src": "cf001e03e5c57dd6"},
    ("c4_f8_8192_rc_silu", "ring_f8_rc_256x256_w2x4_ns5_k64"):
        {"bytes": int((393480.9 * 2.0 + 131206.4) * 1024), "files": RING_F8_SRC, "src": "1b37960b6cd1073e"},
    ("c2_f32_skinny16_rc_silu", "skinnyrc_f32_dma_wk4_cg4_ns2"):
        {"bytes": int((609659.9 * 2.0 + 1024.0) * 1024), "files": SKINNY_RC_SRC, "src": "7ff6f414fc2ebc17"},
    ("s_transpose", "s_transpose"):
        {"bytes": int((524327.0 * 2.0 + 1048910.0) * 1024), "files": TRANSPOSE_SRC, "src": "00f7350d0ac9d4a0"},
    ("s_mhsa", "s_mhsa"):
        {"bytes": int((98401.8 * 2.0 + 65536.0) * 1024), "files": ATTN_SRC, "src": "a4876881c0272702"},
    ("s_lce", "s_lce"):
        {"bytes": int((1590396.8 * 2.0 + 33040.0) * 1024), "files": LCE_SRC, "src": "6afe4dac2e72a9c6"},
    ("s_lce_f32", "s_lce_f32"):
        {"bytes": int((1583509.3 * 2.0 + 32904.0) * 1024), "files": LCE_F32_SRC, "src": "b2d898c0c56d34de"},
}


def kernel_source_hash(files):
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2602_12305_amd", "csrc")
    for f in files:
        h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:16]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--preheat-ms", type=float, default=300.0,
                    help="run the workload back to back for this long before the warm-up steps (clocks at steady state)")
    ap.add_argument("--workload", default="c2_f32_skinny16_silu")
    ap.add_argument("--all", action="store_true", help="also time the other workloads")
    ap.add_argument("--variant", type=int, default=-1, help="force one kernel variant (default: dispatcher)")
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

    from paper_2602_12305_amd import binding as ob
    from paper_2602_12305_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    def to_dev(x):
        return torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x).cuda()

    def preheat(call):
        """Untimed: `call(i)` back to back for --preheat-ms of wall time, before the warm-up steps.  The chip's
        clocks take some 50 ms of sustained work to reach their steady values (the headline workload after 5
        warm-up steps: 0.194 ms per step; after 85 ms of the same work: 0.170 ms, on one board, alternating),
        and the steady state is what this benchmark reports."""
        if args.preheat_ms <= 0:
            return
        t_end = time.perf_counter() + args.preheat_ms * 1e-3
        i = 0
        while time.perf_counter() < t_end:
            for _ in range(16):
                call(i)
                i += 1
            torch.cuda.synchronize()

    if args.copy_gib > 0:
        nbytes = int(args.copy_gib * (1 << 30)) // 16 * 16
        src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        for _ in range(args.warmup):
            ob.optiml_copy_bytes(dst, src, nbytes)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            ob.optiml_copy_bytes(dst, src, nbytes)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        print(json.dumps({"metric": "GB/s of a plain device copy (bytes read + bytes written)", "unit": "GB/s",
                          "value": round(2 * nbytes / (ms * 1e-3) / 1e9, 1), "bytes_read": nbytes,
                          "bytes_written": nbytes, "ms_per_step": round(ms, 5), "steps": args.steps,
                          "frac_of_8TBs": round(2 * nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}))
        return

    def time_workload(name, steps, warmup):
        w = synth.make_workload(name)
        lda, ldb = w.A.shape[-1], w.B.shape[-1]
        sA = w.A.shape[-2] * lda if w.batch > 1 else 0
        sB = w.B.shape[-2] * ldb if w.batch > 1 else 0
        sBias = w.N if w.batch > 1 else 0
        sets = []
        for _ in range(2):
            Cd = torch.empty((w.batch, w.M, w.N), dtype=torch.float32 if w.dtype == 0 else torch.int16, device="cuda")
            sets.append((to_dev(w.A), to_dev(w.B), to_dev(w.bias), Cd))
        probe = (w.batch, w.M, w.N, w.K, sets[0][0], lda, sA, sets[0][1], ldb, sB, sets[0][2], sBias,
                 sets[0][3], w.N, w.M * w.N, w.layout, w.dtype, w.act)
        vid = args.variant if args.variant >= 0 else ob.optiml_select_variant(*probe)

        def step(i):
            Ad, Bd, bd, Cd = sets[i & 1]
            ob.optiml_gemm_epilogue_variant(w.batch, w.M, w.N, w.K, Ad, lda, sA, Bd, ldb, sB, bd, sBias,
                                            Cd, w.N, w.M * w.N, w.layout, w.dtype, w.act, vid)

        preheat(step)
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
        ms = max(wall_ms, dev_ms) / steps          # whole-step time, host view
        kernel_ms = dev_ms / steps                 # HIP events on the launch stream
        gbs = w.algorithmic_bytes / (kernel_ms * 1e-3) / 1e9
        tfl = w.flops / (kernel_ms * 1e-3) / 1e12
        bound = BOUND[name]
        tr = TRAFFIC.get((name, ob.optiml_variant_name(vid)))
        traffic = tr["bytes"] if tr and tr["src"] == kernel_source_hash(tr["files"]) else None
        roof = {"bound": bound,
                "achieved": round(gbs if bound == "hbm" else tfl, 3),
                "peak": PEAK_HBM_GBS if bound == "hbm" else PEAK_TFLOPS[w.dtype],
                "unit": "GB/s" if bound == "hbm" else "TFLOP/s",
                "frac": round((gbs / PEAK_HBM_GBS) if bound == "hbm" else (tfl / PEAK_TFLOPS[w.dtype]), 4),
                "traffic": traffic,
                "kernel": ob.optiml_variant_name(vid),
                "kernel_ms": round(kernel_ms, 5)}
        res = {"workload": name, "variant": ob.optiml_variant_name(vid), "ms_per_step": round(ms, 5),
               "GB/s": round(w.algorithmic_bytes / (ms * 1e-3) / 1e9, 2), "TFLOP/s": round(w.flops / (ms * 1e-3) / 1e12, 3),
               "hbm_frac": round(gbs / PEAK_HBM_GBS, 4), "mfma_frac": round(tfl / PEAK_TFLOPS[w.dtype], 4),
               "dtype": DTYPE_NAME[w.dtype], "roofline": roof}
        return w, sets, res

    def time_stream(name, steps, warmup, with_oracle):
        """One streaming sibling on 2^28 seeded uniform floats (1 GiB per array)."""
        kind, op, reads, writes = STREAMS[name]
        n = STREAM_N
        gen = lambda tag: synth.uniform(7, tag, n >> 16, 1 << 16, -2.0, 2.0).reshape(-1)
        hx = gen("x")
        hy = gen("y") if reads == 2 else None
        xd = torch.from_numpy(hx).cuda()
        yd = torch.from_numpy(hy).cuda() if hy is not None else None
        od = torch.empty(1 if kind == "red" else n, dtype=torch.float32, device="cuda")
        side = 1 << 14                                          # the transpose sees the array as 16384 x 16384
        if kind == "ew":
            step = lambda: ob.optiml_elementwise(n, xd, od, op)
        elif kind == "tr":
            step = lambda: ob.optiml_transpose(side, side, xd, side, od, side, 4)
        else:
            step = lambda: ob.optiml_reduce(n, xd, yd, op, od)
        preheat(lambda i: step())
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            step()
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        dev_ms = e0.elapsed_time(e1)
        ms, kernel_ms = max(wall_ms, dev_ms) / steps, dev_ms / steps
        nbytes = 4 * n * (reads + writes) + (4 if kind == "red" else 0)
        gbs = nbytes / (kernel_ms * 1e-3) / 1e9
        tr = TRAFFIC.get((name, name))
        traffic = tr["bytes"] if tr and tr["src"] == kernel_source_hash(tr["files"]) else None
        res = {"workload": name, "variant": name, "n": n, "ms_per_step": round(ms, 5),
               "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 2), "hbm_frac": round(gbs / PEAK_HBM_GBS, 4), "dtype": "f32",
               "roofline": {"bound": "hbm", "achieved": round(gbs, 3), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                            "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": traffic, "kernel": name,
                            "kernel_ms": round(kernel_ms, 5)}}
        if with_oracle:
            import oracle
            t0 = time.perf_counter()
            if kind == "ew":
                m = 1 << 24                                     # bounded sample: the first 2^24 elements
                ref = oracle.elementwise(hx[:m], op)
                secs = time.perf_counter() - t0
                got = od[:m].cpu().numpy().astype(np.float64)
                err = float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-30)))
                full, sample = secs * (n / m), f"first {m} of {n} elements"
            elif kind == "tr":
                ref = oracle.transpose(hx.reshape(side, side))
                secs = time.perf_counter() - t0
                err = 0.0 if np.array_equal(od.cpu().numpy().reshape(side, side), ref) else 1.0
                full, sample = secs, "whole workload"
            else:
                ref = oracle.reduce(hx, hy, op)
                secs = time.perf_counter() - t0
                err = abs(float(od.item()) - ref) / max(abs(ref), 1e-30)
                full, sample = secs, "whole workload"
            res["cpu_baseline"] = {"value": float(f"{nbytes / 1e9 / full:.4g}"), "unit": "GB/s",
                                   "cores": oracle.num_threads(), "kind": "oracle", "sample": sample,
                                   "seconds": round(secs, 3)}
            res["parity_rel_err"] = float(f"{err:.3e}")
        return res

    def time_rows(name, steps, warmup, with_oracle):
        """Cross-entropy or LayerNorm on a seeded normal array of 1 GiB."""
        rows, cols = ROWS[name]
        hx = synth.normal(8, "x", rows, cols, 0.5, 2.0)
        xd = torch.from_numpy(hx).cuda()
        if name == "s_ce":
            hl = (np.arange(rows, dtype=np.int64) * 7919 % cols).astype(np.int32)
            ld_ = torch.from_numpy(hl).cuda()
            od = torch.empty(1, dtype=torch.float32, device="cuda")
            step = lambda: ob.optiml_cross_entropy(rows, cols, xd, cols, ld_, od)
            nbytes = 4 * rows * cols + 4 * rows + 4
        else:
            od = torch.empty_like(xd)
            step = lambda: ob.optiml_layernorm(rows, cols, xd, od, 1e-5)
            nbytes = 8 * rows * cols
        preheat(lambda i: step())
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            step()
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        dev_ms = e0.elapsed_time(e1)
        ms, kernel_ms = max(wall_ms, dev_ms) / steps, dev_ms / steps
        gbs = nbytes / (kernel_ms * 1e-3) / 1e9
        tr = TRAFFIC.get((name, name))
        traffic = tr["bytes"] if tr and tr["src"] == kernel_source_hash(tr["files"]) else None
        res = {"workload": name, "variant": name, "rows": rows, "cols": cols, "ms_per_step": round(ms, 5),
               "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 2), "hbm_frac": round(gbs / PEAK_HBM_GBS, 4), "dtype": "f32",
               "roofline": {"bound": "hbm", "achieved": round(gbs, 3), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                            "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": traffic, "kernel": name,
                            "kernel_ms": round(kernel_ms, 5)}}
        if with_oracle:
            import oracle
            t0 = time.perf_counter()
            if name == "s_ce":
                ref = oracle.cross_entropy(hx, hl)
                secs = time.perf_counter() - t0
                err = abs(float(od.item()) - ref)
                full, sample = secs, "whole workload"
            else:
                m = max(1, rows // 16)                           # bounded sample: the first sixteenth of the rows
                ref = oracle.layernorm(hx[:m], 1e-5)
                secs = time.perf_counter() - t0
                err = float(np.max(np.abs(od[:m].cpu().numpy().astype(np.float64) - ref)))
                full, sample = secs * (rows / m), f"first {m} of {rows} rows"
            res["cpu_baseline"] = {"value": float(f"{nbytes / 1e9 / full:.4g}"), "unit": "GB/s",
                                   "cores": oracle.num_threads(), "kind": "oracle", "sample": sample,
                                   "seconds": round(secs, 3)}
            res["parity_abs_err"] = float(f"{err:.3e}")
        return res

    def time_mhsa(name, steps, warmup, with_oracle):
        """Multi-head self-attention, bf16 storage, seeded N(0, 1) inputs."""
        batch, N, d, heads = MHSA[name]
        host = [synth.f32_to_bf16_bits(synth.normal(9, tag, N, d, batch=batch)) for tag in ("q", "k", "v")]
        Qd, Kd, Vd = (torch.from_numpy(h.view(np.int16)).cuda() for h in host)
        Od = torch.empty_like(Qd)
        step = lambda: ob.optiml_mhsa(batch, N, d, heads, Qd, Kd, Vd, Od, 1)
        preheat(lambda i: step())
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            step()
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        dev_ms = e0.elapsed_time(e1)
        ms, kernel_ms = max(wall_ms, dev_ms) / steps, dev_ms / steps
        flops = 4.0 * batch * N * N * d                    # two products of 2 N^2 d_k flops per head
        tfl = flops / (kernel_ms * 1e-3) / 1e12
        tr = TRAFFIC.get((name, name))
        traffic = tr["bytes"] if tr and tr["src"] == kernel_source_hash(tr["files"]) else None
        res = {"workload": name, "variant": "mhsa_flash_bf16_dk128", "batch": batch, "N": N, "d_model": d, "heads": heads,
               "ms_per_step": round(ms, 5), "TFLOP/s": round(flops / (ms * 1e-3) / 1e12, 3),
               "mfma_frac": round(tfl / PEAK_TFLOPS[1], 4), "dtype": "bf16",
               "roofline": {"bound": "mfma", "achieved": round(tfl, 3), "peak": PEAK_TFLOPS[1], "unit": "TFLOP/s",
                            "frac": round(tfl / PEAK_TFLOPS[1], 4), "traffic": traffic, "kernel": "mhsa_flash_kernel<128>",
                            "kernel_ms": round(kernel_ms, 5)}}
        if with_oracle:
            import oracle
            t0 = time.perf_counter()
            ref = oracle.mhsa(host[0][:1], host[1][:1], host[2][:1], heads, dtype=oracle.BF16)[0]   # bounded sample
            secs = time.perf_counter() - t0
            got = synth.bf16_bits_to_f32(Od[0].cpu().numpy().view(np.uint16)).astype(np.float64)
            rho = float(np.sqrt(np.mean(ref * ref)))
            err = float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rho)))
            res["cpu_baseline"] = {"value": float(f"{flops / batch / 1e12 / secs:.4g}"), "unit": "TFLOP/s",
                                   "cores": oracle.num_threads(), "kind": "oracle",
                                   "sample": f"sequence 0 of {batch} (all {heads} heads)", "seconds": round(secs, 3)}
            res["parity_e1"] = float(f"{err:.3e}")
        return res

    def time_lce(name, steps, warmup, with_oracle):
        """Contraction + cross-entropy, bf16 storage: A N(0, 1/K) (logits of unit variance), B N(0,1), bias N(0,1)."""
        M, N, K, dt = LCE[name]
        A = synth.to_bits(synth.normal(10, "A", M, K, 0.0, K ** -0.5), dt)
        B = synth.to_bits(synth.normal(10, "B", K, N), dt)
        bias = synth.normal(10, "bias", 1, N)[0]
        labels = ((7919 * np.arange(M)) % N).astype(np.int32)
        Ad, Bd = (torch.from_numpy(h.view(np.int16) if dt else h).cuda() for h in (A, B))
        bd, ld = torch.from_numpy(bias).cuda(), torch.from_numpy(labels).cuda()
        out = torch.empty(2, dtype=torch.float32, device="cuda")
        step = lambda rows=M, o=0: ob.optiml_gemm_cross_entropy(rows, N, K, Ad, K, Bd, N, bd, ld, out[o:], 0, dt)
        assert ob.optiml_gemm_cross_entropy_path(M, N, K, Ad, K, Bd, N, bd, 0, dt) == 0
        preheat(lambda i: step())
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            step()
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        dev_ms = e0.elapsed_time(e1)
        ms, kernel_ms = max(wall_ms, dev_ms) / steps, dev_ms / steps
        flops = 2.0 * M * N * K
        tfl = flops / (kernel_ms * 1e-3) / 1e12
        tr = TRAFFIC.get((name, name))
        traffic = tr["bytes"] if tr and tr["src"] == kernel_source_hash(tr["files"]) else None
        res = {"workload": name, "variant": f"ring_{DTYPE_NAME[dt]}_rr_lse", "M": M, "N": N, "K": K, "ms_per_step": round(ms, 5),
               "TFLOP/s": round(flops / (ms * 1e-3) / 1e12, 3), "mfma_frac": round(tfl / PEAK_TFLOPS[dt], 4),
               "dtype": DTYPE_NAME[dt],
               "loss": float(out[0].item()),
               "roofline": {"bound": "mfma", "achieved": round(tfl, 3), "peak": PEAK_TFLOPS[dt], "unit": "TFLOP/s",
                            "frac": round(tfl / PEAK_TFLOPS[dt], 4), "traffic": traffic,
                            "kernel": ("gemm_ring_kernel" if dt else "gemm_ring_f32_kernel") +
                                      " (log-sum-exp epilogue) + lce_rows_kernel + lce_mean_kernel",
                            "kernel_ms": round(kernel_ms, 5)}}
        if with_oracle:
            import oracle
            m = M // 2                                                 # bounded sample: the first half of the rows
            step(m, 1)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ref = oracle.gemm_cross_entropy(A[:m], B, bias, labels[:m], m, N, K, dtype=dt)
            secs = time.perf_counter() - t0
            res["cpu_baseline"] = {"value": float(f"{flops * (m / M) / 1e12 / secs:.4g}"), "unit": "TFLOP/s",
                                   "cores": oracle.num_threads(), "kind": "oracle", "sample": f"first {m} of {M} rows",
                                   "seconds": round(secs, 3)}
            res["parity_abs_err"] = float(f"{abs(float(out[1].item()) - ref):.3e}")
        return res

    if args.workload in LCE:
        r = time_lce(args.workload, args.steps, args.warmup, not args.no_cpu_baseline)
        out = {"metric": "TFLOP/s of the contraction fused with the cross-entropy", "value": r["TFLOP/s"], "unit": "TFLOP/s",
               "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "preheat_ms": args.preheat_ms, "ms_per_step": r["ms_per_step"],
               "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": r["dtype"], "data": "synthetic",
               "config": {"workload": args.workload, "M": r["M"], "N": r["N"], "K": r["K"]}, "TFLOP/s": r["TFLOP/s"],
               "loss": r["loss"], "roofline": r["roofline"]}
        for k in ("cpu_baseline", "parity_abs_err"):
            if k in r:
                out[k] = r[k]
        print(json.dumps(out))
        return

    if args.workload in MHSA:
        r = time_mhsa(args.workload, args.steps, args.warmup, not args.no_cpu_baseline)
        out = {"metric": "TFLOP/s of multi-head self-attention", "value": r["TFLOP/s"], "unit": "TFLOP/s",
               "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "preheat_ms": args.preheat_ms, "ms_per_step": r["ms_per_step"],
               "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
               "config": {"workload": args.workload, "batch": r["batch"], "N": r["N"], "d_model": r["d_model"],
                          "heads": r["heads"]}, "TFLOP/s": r["TFLOP/s"], "roofline": r["roofline"]}
        for k in ("cpu_baseline", "parity_e1"):
            if k in r:
                out[k] = r[k]
        print(json.dumps(out))
        return

    if args.workload in STREAMS or args.workload in ROWS:
        if args.workload in ROWS:
            r = time_rows(args.workload, args.steps, args.warmup, not args.no_cpu_baseline)
            r["n"] = r["rows"] * r["cols"]
        else:
            r = time_stream(args.workload, args.steps, args.warmup, not args.no_cpu_baseline)
        out = {"metric": "GB/s (algorithmic bytes) of " + args.workload[2:], "value": r["GB/s"], "unit": "GB/s",
               "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "preheat_ms": args.preheat_ms, "ms_per_step": r["ms_per_step"],
               "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
               "config": {"workload": args.workload, "n": r["n"]}, "GB/s": r["GB/s"], "roofline": r["roofline"]}
        for k in ("cpu_baseline", "parity_rel_err", "parity_abs_err"):
            if k in r:
                out[k] = r[k]
        print(json.dumps(out))
        return

    w, sets, head = time_workload(args.workload, args.steps, args.warmup)
    bound = BOUND[args.workload]
    out = {
        "metric": "GB/s (algorithmic bytes) of act(A.B+bias)" if bound == "hbm" else "TFLOP/s of act(A.B+bias)",
        "value": head["GB/s"] if bound == "hbm" else head["TFLOP/s"],
        "unit": "GB/s" if bound == "hbm" else "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "preheat_ms": args.preheat_ms, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": args.workload, "batch": w.batch, "M": w.M, "N": w.N, "K": w.K,
                   "layout": ["rr", "rc", "cr", "cc"][w.layout], "act": ["none", "relu", "gelu_tanh", "silu"][w.act],
                   "variant": head["variant"]},
        "TFLOP/s": head["TFLOP/s"], "GB/s": head["GB/s"],
        "roofline": head["roofline"],
    }

    if not args.no_cpu_baseline:
        import oracle
        # bounded sample of the same workload: whole output if that is about 5e10 multiply-adds
        # or fewer, else seeded sampled entries
        macs = w.flops // 2
        t0 = time.perf_counter()
        if macs <= 8e10:
            ref = oracle.gemm_epilogue(w.A, w.B, w.bias, w.M, w.N, w.K, dtype=w.dtype, act=w.act, layout=w.layout,
                                       batch=w.batch)
            secs = time.perf_counter() - t0
            frac, sample = 1.0, "whole workload"
            got = sets[(args.steps - 1) & 1][3].cpu().numpy()
            idx = None
        else:
            sb, si, sj = synth.sample_entries(w.seed, 1 << 20, w.batch, w.M, w.N)
            ref = oracle.gemm_epilogue_sampled(sb, si, sj, w.A, w.B, w.bias, w.M, w.N, w.K, dtype=w.dtype, act=w.act,
                                               layout=w.layout, batch=w.batch)
            secs = time.perf_counter() - t0
            frac = len(sb) / float(w.batch * w.M * w.N)
            sample = f"{len(sb)} sampled output entries of {w.batch * w.M * w.N}"
            got = sets[(args.steps - 1) & 1][3].cpu().numpy()
            idx = (sb, si, sj)
        if w.dtype != 0:
            got = synth.from_bits(got.view(np.uint16), 1 if w.dtype == 3 else w.dtype)      # E4M3 operands: bf16 result
        got = got.astype(np.float64)
        if idx is not None:
            got = got[idx]
        rho = float(np.sqrt(np.mean(ref * ref)))
        e1 = float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rho)))
        full_secs = secs / frac
        cpu_val = (w.algorithmic_bytes / 1e9 if bound == "hbm" else w.flops / 1e12) / full_secs
        out["cpu_baseline"] = {"value": float(f"{cpu_val:.4g}"), "unit": out["unit"], "cores": oracle.num_threads(),
                               "kind": "oracle", "sample": sample, "seconds": round(secs, 3)}
        out["parity_e1"] = float(f"{e1:.3e}")
    del sets

    if args.all:
        out["workloads"] = {}
        for name in synth.WORKLOADS + synth.BREADTH_WORKLOADS:
            if name == args.workload:
                out["workloads"][name] = head
                continue
            _, s, r = time_workload(name, args.steps, args.warmup)
            del s
            torch.cuda.empty_cache()
            out["workloads"][name] = r
        for name in STREAMS:
            out["workloads"][name] = time_stream(name, args.steps, args.warmup, False)
            torch.cuda.empty_cache()
        for name in ROWS:
            out["workloads"][name] = time_rows(name, args.steps, args.warmup, False)
            torch.cuda.empty_cache()
        for name in MHSA:
            out["workloads"][name] = time_mhsa(name, args.steps, args.warmup, False)
            torch.cuda.empty_cache()
        for name in LCE:
            out["workloads"][name] = time_lce(name, args.steps, args.warmup, False)
            torch.cuda.empty_cache()

    print(json.dumps(out))


if __name__ == "__main__":
    main()
