"""Dispatcher check: for a list of shapes, time every kernel variant that takes the shape and compare the
dispatcher's choice with the fastest one.

    python3 -m paper_2602_12305_amd.dispatch_check [--set mid|other|batched|ragged|odd|rounds|stream|six|quick] [--steps N]

Prints one line per case (shape, the dispatcher's variant and its time, the fastest variant and its time, the
ratio) and a summary.  Inputs are N(0,1) (8-bit operands: random bytes below 120); nothing is checked for
correctness here, the parity tests do that.  The guarded fallback is left out above 50 GFLOP (minutes per call).
"""
import argparse
import sys
import time

import torch

from . import binding as ob

DT_NAME = {0: "f32", 1: "bf16", 2: "f16", 3: "e4m3", 4: "e2m1", 5: "e5m2", 6: "e2m3", 7: "e3m2"}
LAYOUT_NAME = {0: "rr", 1: "rc", 2: "cr", 3: "cc"}
TORCH_DT = {0: torch.float32, 1: torch.bfloat16, 2: torch.float16}

MID = [(1, 64, 4096, 4096), (1, 128, 8192, 8192), (1, 256, 4096, 4096), (1, 512, 2048, 2048), (1, 1024, 1024, 1024),
       (1, 2048, 2048, 2048), (1, 32, 16384, 1024), (1, 4096, 512, 4096), (1, 512, 8192, 256), (8, 512, 512, 512),
       (1, 8, 4096, 4096), (1, 48, 8192, 8192), (1, 1, 16384, 16384), (1, 3000, 3000, 3000), (1, 4096, 4096, 4096),
       (1, 1536, 1536, 1536), (1, 96, 2048, 2048), (4, 128, 1024, 1024), (1, 64, 16384, 16384), (1, 200, 5120, 1280),
       (1, 768, 3072, 768), (1, 2048, 8192, 1024), (16, 64, 64, 64), (1, 24, 1024, 8192)]
OTHER = [(1, 64, 4096, 4096), (1, 256, 4096, 4096), (1, 1024, 1024, 1024), (1, 2048, 2048, 2048), (1, 4096, 4096, 4096),
         (1, 32, 16384, 1024), (1, 512, 8192, 256), (8, 512, 512, 512), (1, 8, 4096, 4096), (1, 3008, 3008, 3008)]
BATCHED = [(64, 128, 128, 64), (256, 64, 64, 128), (16, 1024, 1024, 128), (4, 2048, 2048, 2048), (32, 256, 256, 256),
           (8, 16, 4096, 4096), (128, 512, 64, 512), (2, 4096, 4096, 1024)]
# up to a few blocks of 16 rows over a large B: the streaming kernels' ground
STREAM = [(16, 16384, 16384), (8, 16384, 16384), (1, 16384, 16384), (16, 8192, 8192), (16, 4096, 4096), (16, 32768, 8192),
          (16, 8192, 32768), (16, 16384, 4096), (16, 2048, 2048), (16, 1024, 1024), (16, 12288, 4096), (4, 5120, 5120),
          (16, 28672, 8192), (16, 65536, 4096), (16, 1024, 65536), (16, 16000, 16000), (13, 10000, 12000), (32, 16384, 16384),
          (32, 4096, 4096), (32, 8192, 8192), (64, 8192, 8192), (128, 4096, 4096), (128, 2048, 2048), (256, 2048, 2048),
          (64, 2048, 8192), (96, 1024, 4096), (16, 16640, 16384), (16, 20480, 8192), (16, 24576, 8192), (16, 10240, 16384)]
SETS = {
    "stream": [(dt, lay, 1) + s for dt, lay in ((0, 0), (1, 0), (1, 1)) for s in STREAM],
    "mid": [(dt, lay) + s for dt in (1, 0) for lay in (0, 1) for s in MID],
    "other": [(dt, lay) + s for dt, lay in ((3, 1), (3, 0), (1, 2), (1, 3), (0, 2), (0, 3)) for s in OTHER],
    "batched": [(dt, lay) + s for dt, lay in ((1, 0), (1, 1), (0, 0), (0, 1), (2, 0)) for s in BATCHED],
    # K (and the row pitch) not a whole number of k-tiles
    "ragged": [(dt, lay, 1, n, n, n) for dt in (1, 2, 0) for lay in (0, 1) for n in (1000, 1496, 3000)] +
              [(3, 1, 1, 1008, 1008, 1008), (3, 1, 1, 3024, 3024, 3024), (1, 0, 1, 64, 4096, 4104), (0, 1, 1, 48, 8192, 8196)],
    # odd sizes and pitches: nothing but the copy path (xpad) and the fallback takes these
    "odd": [(dt, lay, 1) + s for dt in (1, 0) for lay in (0, 1, 3)
            for s in ((1025, 1031, 2051), (4097, 4097, 4097), (301, 395, 203), (17, 4099, 4099), (513, 515, 517))],
    # tile counts a little over a multiple of the CU count (and one well over): the last round of tiles
    "rounds": [(dt, lay, 1) + s for dt, lay in ((1, 0), (1, 1), (2, 0))
               for s in ((4352, 4352, 4352), (4352, 4352, 8192), (4104, 4104, 4104), (4352, 4096, 4096), (4608, 4352, 4096),
                         (8448, 8448, 4096), (4352, 4352, 2048))],
    # 6-bit operands (dense), k contiguous in both: the streaming kernels up to 16 rows, else the copy into slots + ring kernel
    "six": [(dt, 1, 1) + s for dt in (6, 7)
            for s in ((16, 16384, 16384), (16, 28672, 8192), (16, 8192, 8192), (4, 8192, 8192), (16, 4096, 4096), (16, 512, 16384),
                      (16, 16384, 1024), (8, 2048, 2048), (16, 16384, 16416), (16, 4100, 4128), (16, 1030, 4224), (13, 10016, 12032),
                      (64, 64, 1024), (300, 520, 228), (300, 520, 100), (512, 512, 512), (1024, 1024, 1024), (2048, 2048, 2048),
                      (4096, 4096, 4096), (8192, 8192, 8192), (17, 4096, 4096), (64, 8192, 8192), (32, 16384, 16384), (128, 8192, 8192),
                      (128, 2048, 2048), (48, 16384, 4096), (129, 8192, 8192))],
    "quick": [(1, 1, 1, 64, 4096, 4096), (0, 1, 1, 64, 4096, 4096), (1, 2, 1, 64, 4096, 4096), (0, 0, 1, 8, 4096, 4096),
              (1, 0, 1, 2048, 2048, 2048), (0, 0, 1, 4096, 512, 4096)],
}


def _time(prob, vid, steps, preheat_ms=20.0):
    # untimed calls for preheat_ms first: clocks near their steady state (see bench.py)
    t_end = time.perf_counter() + preheat_ms * 1e-3
    while True:
        for _ in range(3):
            ob.optiml_gemm_epilogue_variant(*prob, vid)
        torch.cuda.synchronize()
        if time.perf_counter() >= t_end:
            break
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        ob.optiml_gemm_epilogue_variant(*prob, vid)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps * 1e3            # microseconds


def check(dt, lay, b, M, N, K, steps=0, names=None):
    """(name of the dispatcher's variant, its us, name of the fastest variant, its us)."""
    names = names or ob.variant_names()
    num, den = {4: (1, 2), 6: (3, 4), 7: (3, 4)}.get(dt, (1, 1))     # stored bytes per element of the sub-byte types
    if dt >= 3:
        def mk(shape):
            return torch.randint(0, 120, shape[:-1] + (shape[-1] * num // den,), device="cuda", dtype=torch.uint8)
    else:
        def mk(shape):
            return torch.randn(shape, device="cuda", dtype=TORCH_DT[dt])
    A = mk((b, K, M) if lay & 2 else (b, M, K))
    B = mk((b, N, K) if lay & 1 else (b, K, N))
    bias = torch.randn((b, N), device="cuda", dtype=torch.float32)
    C = torch.empty((b, M, N), device="cuda", dtype=torch.bfloat16 if dt >= 3 else TORCH_DT[dt])
    lda, ldb = A.shape[-1] * den // num, B.shape[-1] * den // num
    prob = (b, M, N, K, A, lda, A.shape[-2] * lda, B, ldb, B.shape[-2] * ldb, bias, N, C, N, M * N, lay, dt, 3)
    pick = ob.optiml_select_variant(*prob)
    flops = 2.0 * b * M * N * K
    steps = steps or max(3, min(50, int(2e11 / max(flops, 1e9))))
    best = None
    t_pick = None
    only_fallback_left = names[pick] in ("xpad", "generic_64x64")
    for i, n in enumerate(names):
        if n.startswith("generic") and flops > 5e10 and i != pick and not only_fallback_left:
            continue
        if ob.optiml_variant_supports(i, *prob) != 0:
            continue
        t = _time(prob, i, steps)
        if i == pick:
            t_pick = t
        if best is None or t < best[0]:
            best = (t, n)
    return names[pick], t_pick, best[1], best[0]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--set", default="mid", choices=sorted(SETS))
    ap.add_argument("--steps", type=int, default=0, help="timed calls per variant (default: by size)")
    a = ap.parse_args()
    if not torch.cuda.is_available():
        sys.exit("dispatch_check needs the GPU")
    names = ob.variant_names()
    ratios = []
    for dt, lay, b, M, N, K in SETS[a.set]:
        pn, pt, bn, bt = check(dt, lay, b, M, N, K, a.steps, names)
        ratios.append(pt / bt)
        print(f"{DT_NAME[dt]:5s} {LAYOUT_NAME[lay]} {b}x{M}x{N}x{K}: {pn} {pt:.1f} us | fastest {bn} {bt:.1f} us | "
              f"ratio {pt / bt:.2f}", flush=True)
    ratios.sort()
    within = sum(r <= 1.10 for r in ratios)
    print(f"{len(ratios)} cases: {within} within 10 % of the fastest variant, worst ratio {ratios[-1]:.2f}")


if __name__ == "__main__":
    main()
