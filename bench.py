"""Benchmark of the swizzled bf16 GEMM on one MI355X.

One "step" is one whole pass of the hot path: a single swz_gemm launch (PID remap, raster
decode, global->LDS staging, MFMA loop, epilogue) over the 4096^3 workload, inputs resident
in HBM.  Prints ONE JSON line.  `value` is the throughput of the swizzled mapping (XCD
renumbering + grouped-M raster); the round-robin and XCD-only mappings, timed the same way in
the same run, are reported beside it, as is the 8192^3 workload.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0        # MI355X dense bf16 MFMA, published (256 CUs x 4 SIMDs x 1024 flop/clk x 2.4 GHz)

# HBM/fabric bytes per launch of the swizzled kernel from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE (KiB per dispatch), each scaled by what the same counter reads for the library's
# plain 1 GiB copy kernel (FETCH_SIZE reads 0.5x the bytes copied, WRITE_SIZE 1.0x).  Valid only
# for the kernel source whose hash is recorded here; any other kernel reports null.
TRAFFIC = {
    "kernel_sha256": "10b69e0b1b7bd1b679568ad5b5be53d185f5b8cdb0704f55d68931199d69d3a9",
    # FETCH_SIZE 98985 KiB x 2.000 + WRITE_SIZE 34304 KiB x 1.000 per dispatch (profiles/gemm_cfg2_4096.txt)
    "cfg2_4096": {"xcd_groupm": {"fetch_bytes": 202716009, "write_bytes": 35127291, "total_bytes": 237843300,
                                 "algorithmic_min_bytes": 100663296}},
}


def kernel_hash() -> str:
    h = hashlib.sha256()
    for name in ("gemm_kernel.h", "pid_decode.h"):
        with open(os.path.join(ROOT, "paper_2508_20258_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def time_mode(swz, torch, a, b, c, mode, steps, warmup, **params):
    """Average launch duration in ms: events recorded on the stream the kernel is launched on."""
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        swz.gemm(a, b, c, mode=mode, stream=stream, **params)
    torch.cuda.synchronize()
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record(stream)
    for _ in range(steps):
        swz.gemm(a, b, c, mode=mode, stream=stream, **params)
    stop.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return start.elapsed_time(stop) / steps, wall_ms / steps


def to_device(torch, np, bits):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def cpu_baseline(a_bits, b_bits, rows):
    """The oracle as it stands, on the host cores, on the first `rows` rows of the same workload."""
    from oracle import gemm_ref
    threads = gemm_ref.num_threads()
    gemm_ref.gemm(a_bits[:8], b_bits)                       # page everything in
    t0 = time.perf_counter()
    gemm_ref.gemm(a_bits[:rows], b_bits)
    dt = time.perf_counter() - t0
    K, N = b_bits.shape
    what = "the whole workload" if rows == a_bits.shape[0] else f"rows 0..{rows - 1} of A against all of B"
    return dict(value=2.0 * rows * N * K / dt / 1e12, unit="TFLOP/s", cores=threads, kind="oracle",
                sample=f"{what} ({rows}x{N}x{K}), fp64 triple loop with OpenMP over rows, {dt:.1f} s")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2_4096")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the 8192^3 workload and the vendor-BLAS context line")
    ap.add_argument("--cpu-rows", type=int, default=0, help="rows of A the oracle is timed on (0 = all)")
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
    a, b = to_device(torch, np, a_bits), to_device(torch, np, b_bits)
    c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    plan = swz.gemm_plan(M, N, K)
    flops = 2.0 * M * N * K

    def pct(t):
        return 100.0 * t / PEAK_BF16_TFLOPS

    per_mode = {}
    for name in ("rr", "xcd", "xcd_groupm"):
        ms, _ = time_mode(swz, torch, a, b, c, swz.MODES[name], max(args.steps // 4, 1), args.warmup)
        per_mode[name] = dict(ms=ms, tflops=flops / ms / 1e9, pct_mfma_peak=pct(flops / ms / 1e9))
    # the paper's own launch style (as many workgroups as compute units, tile loop), unswizzled and swizzled
    for name in ("rr", "xcd_groupm"):
        ms, _ = time_mode(swz, torch, a, b, c, swz.MODES[name], max(args.steps // 4, 1), args.warmup, persistent=1)
        per_mode["persistent_" + name] = dict(ms=ms, tflops=flops / ms / 1e9, pct_mfma_peak=pct(flops / ms / 1e9))
    # the headline run: exactly `steps` timed launches of the swizzled kernel
    ms, wall_ms = time_mode(swz, torch, a, b, c, swz.MODE_XCD_GROUPM, args.steps, args.warmup)
    tflops = flops / ms / 1e9

    traffic, traffic_detail = None, None
    rec = TRAFFIC.get(args.workload, {}).get("xcd_groupm")
    if rec is not None and TRAFFIC["kernel_sha256"] == kernel_hash():
        traffic, traffic_detail = rec["total_bytes"], rec

    out = {
        "metric": "bf16 GEMM TFLOP/s + % MFMA peak + L2 hit rate, swizzled vs round-robin PID",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: M={M} N={N} K={K}, tile {plan['bm']}x{plan['bn']}x{plan['bk']}, "
                               f"grid {plan['grid_m']}x{plan['grid_n']}, num_xcd {plan['num_xcd']}, group_m {plan['group_m']}",
                   "mode": "xcd_groupm"},
        "pct_mfma_peak": pct(tflops),
        "wall_ms_per_step": wall_ms,
        "modes": per_mode,
        "swizzled_over_rr": per_mode["xcd_groupm"]["tflops"] / per_mode["rr"]["tflops"],
        "l2_hit_rate": "not measurable inside this process; rocprofv3 TCC_HIT/TCC_MISS summaries per workload and mode are under profiles/",
        "roofline": {"bound": "mfma", "achieved": tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops / PEAK_BF16_TFLOPS, "traffic": traffic},
        "traffic_detail": traffic_detail,
    }

    if not args.no_extras:
        # context, not the headline: what the vendor BLAS behind torch.matmul does on the same bits
        for _ in range(10):
            torch.matmul(a, b, out=c)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(50):
            torch.matmul(a, b, out=c)
        e1.record()
        torch.cuda.synchronize()
        out["context_vendor_blas_tflops"] = flops / (e0.elapsed_time(e1) / 50) / 1e9
        # the large square workload, same launch path
        big = "cfg3_8192"
        bc = si.CONFIGS[big]
        a3b, b3b = si.config_inputs(big)
        a3, b3 = to_device(torch, np, a3b), to_device(torch, np, b3b)
        c3 = torch.empty((bc["M"], bc["N"]), dtype=torch.bfloat16, device="cuda")
        f3 = 2.0 * bc["M"] * bc["N"] * bc["K"]
        extra = {}
        for name in ("rr", "xcd", "xcd_groupm"):
            m3, _ = time_mode(swz, torch, a3, b3, c3, swz.MODES[name], 30, 5)
            extra[name] = dict(ms=m3, tflops=f3 / m3 / 1e9, pct_mfma_peak=pct(f3 / m3 / 1e9))
        out["other_workloads"] = {big: extra}
        del a3, b3, c3

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(a_bits, b_bits, args.cpu_rows or M)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
