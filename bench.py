"""Benchmark of the swizzled bf16 GEMM on one MI355X.

One "step" is one whole pass of the hot path: a single swz_gemm launch (PID remap, raster
decode, global->LDS staging, MFMA loop, epilogue) over the 4096^3 workload, inputs resident
in HBM.  Prints ONE JSON line.  `value` is the throughput of the swizzled mapping (XCD
renumbering + grouped-M raster) over exactly --steps timed launches; the round-robin and
XCD-only mappings and the persistent launch style, timed interleaved in the same run, are
reported beside it ("modes"), and the same comparison for the other four workloads
("other_workloads": 512^3, 8192^3, the skinny 16384x2048x8192 and the ragged 10000x7000x4096).
L2 hit rates (total and per XCD) and HBM/fabric bytes cannot be read inside this process: they
are the rocprofv3 counters `harness profile --record` stored for exactly these kernel sources
(null when the sources have changed since).  Under "other_kernels": the transpose / softmax /
layer normalisation kernels (HBM-bound; not part of `value`).
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

PEAK_BF16_TFLOPS = 2500.0        # MI355X dense bf16 MFMA, published (256 CUs x 4 SIMDs x 1024 flop/clk x 2.4 GHz)

PER_PASS = 20                    # launches per timing sample of the mapping comparison, whatever --steps is


def recorded(workload):
    """rocprofv3 counters stored for this workload and the kernel sources as they are now (else None):
    per mapping, L2 hit rate (TCC_HIT/(TCC_HIT+TCC_MISS), total and per XCD) and HBM/fabric bytes per launch
    (FETCH_SIZE, WRITE_SIZE in KiB per dispatch, each scaled by what the same counter reads for the
    library's plain 1 GiB copy kernel)."""
    from paper_2508_20258_amd import harness
    return harness.recorded_counters(workload)


def l2_hit_rates(rec):
    if not rec:
        return None
    return {mode: {"total": r["l2_hit_pct"], "per_xcd": r["l2_hit_pct_per_xcd"], "panel_model": r["model_hit_pct"]}
            for mode, r in rec.items()}


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


def compare_mappings(swz, torch, a, b, c, variants, per_pass, warmup, flops, passes=9):
    """Time several mappings interleaved (passes over all of them, median per mapping) after a common
    warm-up, so that clock ramp-up and drift do not favour whichever is measured last; the order inside a
    pass rotates, so that no mapping always runs right behind the same neighbour."""
    def mode_of(name):
        return swz.MODES[name.replace("persistent_", "")]
    for name, params in variants:
        time_mode(swz, torch, a, b, c, mode_of(name), warmup, warmup, **params)
    samples = {name: [] for name, _ in variants}
    for p in range(passes):
        k = p % len(variants)
        for name, params in variants[k:] + variants[:k]:
            ms, _ = time_mode(swz, torch, a, b, c, mode_of(name), per_pass, 2, **params)
            samples[name].append(ms)
    out = {}
    for name, _ in variants:
        ms = sorted(samples[name])[passes // 2]
        t = flops / ms / 1e9
        out[name] = dict(ms=ms, tflops=t, pct_mfma_peak=100.0 * t / PEAK_BF16_TFLOPS)
    return out


def time_calls(torch, fn, n=20):
    """Average duration in us of n back-to-back calls of fn() on the current stream (after two warm-up calls)."""
    for _ in range(2):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / n


def measured_mfma_peak(swz, torch):
    """Sustained rate of back-to-back independent MFMAs on register operands (no memory traffic), all CUs busy:
    what the matrix cores deliver on this device at the clock the data lets it hold."""
    out = torch.empty(512 * 1024, dtype=torch.float32, device="cuda")
    res = {}
    for name, rnd in (("random_operands", True), ("zero_operands", False)):
        swz.mfma_peak(out, 2000, rnd)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flop = swz.mfma_peak(out, 20000, rnd)
        e1.record()
        torch.cuda.synchronize()
        res[name] = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
    return res


def other_kernels(swz, torch):
    """The paper's other kernels built here (transpose, row softmax, layer normalisation): round-robin against the
    remapped program ids, GB/s of the algorithmic 4*M*N bytes against the 8 TB/s HBM roofline, and against the rate
    the library's plain copy kernel reaches in this same run on the same amount of data."""
    res = {}

    def entry(us, m, n, copy_gbs=None):
        gbs = 4.0 * m * n / (us * 1e-6) / 1e9
        e = dict(us=us, gb_per_s=gbs, frac_hbm_peak=gbs / 8000.0)
        if copy_gbs:
            e["frac_of_plain_copy"] = gbs / copy_gbs
        return e

    m = n = 16384
    x = torch.randint(-32768, 32767, (m, n), dtype=torch.int16, device="cuda").view(torch.bfloat16)
    y = torch.empty((n, m), dtype=torch.bfloat16, device="cuda")
    us = time_calls(torch, lambda: swz.copy_bytes(x, y))
    copy_gbs = 4.0 * m * n / (us * 1e-6) / 1e9
    res[f"plain_copy_{m}x{n}"] = entry(us, m, n)
    for tile in (64, 128, 32):
        for mode in ("rr", "xcd_groupm", "xcd_groupm_skew"):
            us = time_calls(torch, lambda: swz.transpose(x, y, tile=tile, mode=swz.MODES[mode]))
            res[f"transpose_{m}x{n}_tile{tile}_{mode}"] = entry(us, m, n, copy_gbs)
    del x, y
    # 32768 x 16384: 1 GiB in, 1 GiB out, beyond what the 256 MB memory-side cache can hold between launches;
    # the smaller cases are partly served from it and are listed for the mapping comparison only
    for (m, n, chunks) in ((32768, 16384, 1), (1024, 65536, 8), (8192, 8192, 1)):
        x = (torch.randn((m, n), device="cuda") * 2.0).to(torch.bfloat16)
        y = torch.empty_like(x)
        g = torch.rand(n, device="cuda").to(torch.bfloat16)
        b = torch.rand(n, device="cuda").to(torch.bfloat16)
        for mode in ("rr", "xcd"):
            us = time_calls(torch, lambda: swz.softmax(x, y, chunks=chunks, mode=swz.MODES[mode]))
            res[f"softmax_{m}x{n}_chunks{chunks}_{mode}"] = entry(us, m, n)
            us = time_calls(torch, lambda: swz.layernorm(x, g, b, y, eps=1e-5, chunks=chunks, mode=swz.MODES[mode]))
            res[f"layernorm_{m}x{n}_chunks{chunks}_{mode}"] = entry(us, m, n)
        del x, y
    return res


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

    variants = [("rr", {}), ("xcd", {}), ("xcd_groupm", {}),
                # grouped raster without the XCD renumbering: what a kernel unaware of the chiplets would use
                ("groupm", {}),
                # the paper's own launch style (as many workgroups as compute units, tile loop)
                ("persistent_rr", dict(persistent=1)), ("persistent_xcd_groupm", dict(persistent=1))]
    per_mode = compare_mappings(swz, torch, a, b, c, variants, PER_PASS, max(args.warmup, PER_PASS), flops)
    # the headline run: exactly `steps` timed launches of the swizzled kernel
    ms, wall_ms = time_mode(swz, torch, a, b, c, swz.MODE_XCD_GROUPM, args.steps, args.warmup)
    tflops = flops / ms / 1e9

    rec = recorded(args.workload)
    traffic, traffic_detail = None, None
    if rec and "xcd_groupm" in rec:
        r = rec["xcd_groupm"]
        traffic = r["fetch_bytes"] + r["write_bytes"]
        traffic_detail = {"fetch_bytes": r["fetch_bytes"], "write_bytes": r["write_bytes"], "total_bytes": traffic,
                          "algorithmic_min_bytes": 2 * (M * K + K * N + M * N),
                          "fetch_bytes_by_mode": {m: v["fetch_bytes"] for m, v in rec.items()}}

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
        "l2_hit_rate": l2_hit_rates(rec),
        "l2_hit_rate_source": "rocprofv3 --pmc TCC_HIT TCC_MISS on this kernel source (harness profile --record); percent; "
                              "null when the kernel sources differ from the profiled ones",
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
        # the other four workloads (small, large square, skinny projection-shaped, ragged), same launch path,
        # same interleaved comparison; launches per sample sized so that a sample lasts a few milliseconds
        out["other_workloads"] = {}
        for other in [w for w in si.CONFIGS if w != args.workload]:
            oc = si.CONFIGS[other]
            ab, bb = si.config_inputs(other)
            a3, b3 = to_device(torch, np, ab), to_device(torch, np, bb)
            c3 = torch.empty((oc["M"], oc["N"]), dtype=torch.bfloat16, device="cuda")
            f3 = 2.0 * oc["M"] * oc["N"] * oc["K"]
            n3 = 200 if f3 < 1e10 else PER_PASS if f3 < 2e11 else 8
            res = compare_mappings(swz, torch, a3, b3, c3, variants, n3, n3, f3)
            res["l2_hit_rate"] = l2_hit_rates(recorded(other))
            res["swizzled_over_rr"] = res["xcd_groupm"]["tflops"] / res["rr"]["tflops"]
            out["other_workloads"][other] = res
            del a3, b3, c3, ab, bb

    if not args.no_extras:
        out["other_kernels"] = other_kernels(swz, torch)
        peak = measured_mfma_peak(swz, torch)
        out["measured_mfma_peak_tflops"] = peak
        out["pct_measured_mfma_peak"] = 100.0 * tflops / peak["random_operands"]

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(a_bits, b_bits, args.cpu_rows or M)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
