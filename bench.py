"""Benchmark of the swizzled bf16 GEMM on one MI355X.

One "step" is one whole pass of the hot path: a single swz_gemm launch (PID remap, raster
decode, staging, MFMA loop, epilogue) over the 4096^3 workload with inputs resident in HBM.
Prints ONE JSON line.  `value` is the swizzled (XCD renumbering + grouped-M) throughput; the
round-robin and XCD-only figures measured in the same run are reported beside it.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0        # MI355X dense bf16 MFMA, published


def time_mode(swz, torch, a, b, c, mode, steps, warmup):
    """Average launch duration in ms, from events on the stream the kernel is launched on."""
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        swz.gemm(a, b, c, mode=mode, stream=stream)
    torch.cuda.synchronize()
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record(stream)
    for _ in range(steps):
        swz.gemm(a, b, c, mode=mode, stream=stream)
    stop.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return start.elapsed_time(stop) / steps, wall_ms / steps


def cpu_baseline(si, a_bits, b_bits, rows):
    """The oracle as it stands, on the host cores, on the first `rows` rows of the same workload."""
    from oracle import gemm_ref
    threads = gemm_ref.num_threads()
    sub = a_bits[:rows]
    gemm_ref.gemm(sub[:8], b_bits)                       # page everything in
    t0 = time.perf_counter()
    gemm_ref.gemm(sub, b_bits)
    dt = time.perf_counter() - t0
    K, N = b_bits.shape
    return dict(value=2.0 * rows * N * K / dt / 1e12, unit="TFLOP/s", cores=threads, kind="oracle",
                sample=f"rows 0..{rows - 1} of the same A against all of B ({rows}x{N}x{K}), fp64 triple loop, {dt:.1f} s")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2_4096")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=768)
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this path uses no second device (run with --gpus 1)")

    import numpy as np
    import torch

    import paper_2508_20258_amd as swz
    import seeded_inputs as si

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = si.CONFIGS[args.workload]
    M, N, K = cfg["M"], cfg["N"], cfg["K"]
    a_bits, b_bits = si.config_inputs(args.workload)
    a = torch.from_numpy(a_bits.view(np.int16)).cuda().view(torch.bfloat16)
    b = torch.from_numpy(b_bits.view(np.int16)).cuda().view(torch.bfloat16)
    c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    plan = swz.gemm_plan(M, N, K)
    flops = 2.0 * M * N * K

    per_mode = {}
    for name in ("rr", "xcd", "xcd_groupm"):
        ms, _ = time_mode(swz, torch, a, b, c, swz.MODES[name], max(args.steps // 4, 1), args.warmup)
        per_mode[name] = dict(ms=ms, tflops=flops / ms / 1e9)
    # the headline run: exactly `steps` timed launches of the swizzled kernel
    ms, wall_ms = time_mode(swz, torch, a, b, c, swz.MODE_XCD_GROUPM, args.steps, args.warmup)
    tflops = flops / ms / 1e9

    out = {
        "metric": "bf16 GEMM TFLOP/s + % MFMA peak + L2 hit rate, swizzled vs round-robin PID",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: M={M} N={N} K={K}, tile {plan['bm']}x{plan['bn']}x{plan['bk']}, "
                               f"grid {plan['grid_m']}x{plan['grid_n']}, num_xcd {plan['num_xcd']}, group_m {plan['group_m']}",
                   "mode": "xcd_groupm"},
        "pct_mfma_peak": 100.0 * tflops / PEAK_BF16_TFLOPS,
        "wall_ms_per_step": wall_ms,
        "modes": {k: {"ms": v["ms"], "tflops": v["tflops"], "pct_mfma_peak": 100.0 * v["tflops"] / PEAK_BF16_TFLOPS}
                  for k, v in per_mode.items()},
        "swizzled_over_rr": per_mode["xcd_groupm"]["tflops"] / per_mode["rr"]["tflops"],
        "roofline": {"bound": "mfma", "achieved": tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops / PEAK_BF16_TFLOPS, "traffic": None},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(si, a_bits, b_bits, min(args.cpu_rows, M))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
