"""Profiling harness for the swizzled GEMM: the program that runs under rocprofv3, the reader that
turns rocprofv3's CSV / JSON output into the summaries kept with the measurements, and the
candidate search of the paper's optimisation loop without the LLM.

    python -m paper_2508_20258_amd.harness run --workload cfg2_4096 --mode xcd_groupm --launches 20
    python -m paper_2508_20258_amd.harness profile --workload cfg2_4096 --out <dir> [--record]
    python -m paper_2508_20258_amd.harness rank --workload cfg4_skinny
    python -m paper_2508_20258_amd.harness clocks --workload cfg2_4096 --mode xcd_groupm
    python -m paper_2508_20258_amd.harness copy --mib 1024 --launches 3
    python -m paper_2508_20258_amd.harness transpose --m 16384 --n 16384 --tile 32 --mode rr
    python -m paper_2508_20258_amd.harness rows --op softmax --m 8192 --n 8192 --chunks 8 --mode xcd
    python -m paper_2508_20258_amd.harness peak
    python -m paper_2508_20258_amd.harness summarize <rocprofv3 output dir>

`run` launches one mapping mode of one workload: untimed warm-up launches worth `--warmup-ms` of GPU
time, then `--launches` timed ones; in a kernel trace of such a run the timed launches are the last
`--launches` dispatches of the kernel, which is what `profile` averages.  The warm-up has to outlast
the power controller's transient: a device coming out of idle runs this kernel at boost clocks for
about 2 ms (92 us per 4096^3 launch), is then throttled well below its sustained rate (up to 130 us
around 3-4 ms) and settles after about 10 ms; numbers taken inside that window are not the
sustained ones.  `copy` launches the plain copy kernel of known HBM
traffic, against which FETCH_SIZE / WRITE_SIZE are scaled.  `profile` runs every rocprofv3 pass for
the three mappings of a workload as child processes and prints the table kept under profiles/;
`--record` also stores the counters, keyed by the SHA-256 of the kernel sources, where bench.py
finds them.  `rank` is the non-LLM core of the paper's loop (Methodology, step 4): it lists
candidate remaps (mapping mode x group_m x tile), predicts each one's L2 reuse with a panel-count
model evaluated on the library's own swz_pid_map, profiles them in that order, checks each one (a
candidate whose C differs bitwise from the round-robin launch, or whose PID map is not a
permutation, is a broken remap and is dropped), ranks the rest by measured L2 hit rate and names
the best.  `profile` and `rank` start child processes and never touch the GPU themselves.
The metric the paper ranks remaps by is the L2 hit rate (SwizzlePerf, Methodology step 2 and 4):
here  TCC_HIT / (TCC_HIT + TCC_MISS), from the summed TCC counters.
"""
from __future__ import annotations

import argparse
import csv
import glob
import os
import sys
from collections import defaultdict

HERE = os.path.dirname(os.path.abspath(__file__))
MODE_NAMES = ["rr", "xcd", "xcd_groupm", "groupm", "rr_skew", "xcd_skew", "xcd_groupm_skew", "groupm_skew"]


def _inputs(workload):
    """Seeded inputs of a workload on the device.  The bit patterns are kept in a file under TMPDIR between the
    many short child processes of `profile` and `rank` (generating 8192^2 matrices takes longer than a pass)."""
    import tempfile

    import numpy as np
    import torch

    import seeded_inputs as si
    cache = os.path.join(tempfile.gettempdir(), f"swz_inputs_{workload}_{os.getuid()}.npz")
    a_bits = b_bits = None
    if os.path.exists(cache):
        try:
            with np.load(cache, allow_pickle=False) as z:
                a_bits, b_bits = z["a"], z["b"]
        except Exception:
            a_bits = b_bits = None
    cfg = si.CONFIGS[workload]
    if a_bits is None or a_bits.shape != (cfg["M"], cfg["K"]) or b_bits.shape != (cfg["K"], cfg["N"]):
        a_bits, b_bits = si.config_inputs(workload)
        try:
            tmp = cache + f".{os.getpid()}.tmp.npz"
            np.savez(tmp, a=a_bits, b=b_bits)
            os.replace(tmp, cache)
        except OSError:
            pass
    a = torch.from_numpy(a_bits.view(np.int16)).cuda().view(torch.bfloat16)
    b = torch.from_numpy(b_bits.view(np.int16)).cuda().view(torch.bfloat16)
    return a, b


def kernel_hash() -> str:
    """SHA-256 of the GEMM kernel sources: recorded counters are only valid for the kernel they were taken on."""
    import hashlib
    h = hashlib.sha256()
    for name in ("gemm_kernel.h", "pid_decode.h"):
        with open(os.path.join(HERE, "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def panel_model(tile_of_wg, grid_n, num_xcd, slots):
    """Lock-step panel count of a PID map (tile_of_wg[w] = pm*grid_n + pn, e.g. from swz_pid_map).

    Workgroup w runs on XCD w mod num_xcd; an XCD works on `slots` tiles at a time, in dispatch order,
    and those advance through K together, each asking for one A row-panel and one B column-panel per
    K step.  A panel a co-resident tile also asks for is served by the XCD's L2.  Returns
    (predicted hit rate, distinct panels fetched, panels requested)."""
    requested = distinct = 0
    for x in range(num_xcd):
        mine = [int(t) for t in tile_of_wg[x::num_xcd]]
        for s in range(0, len(mine), slots):
            batch = mine[s:s + slots]
            requested += 2 * len(batch)
            distinct += len({t // grid_n for t in batch}) + len({t % grid_n for t in batch})
    return (1.0 - distinct / requested if requested else 0.0), distinct, requested


def co_resident_tiles_per_xcd(tile, compute_units, num_xcd):
    """Tiles one XCD works on at a time: a 256-wide tile fills a CU's LDS, two 128-wide ones fit."""
    return (compute_units // num_xcd) * (1 if tile >= 256 else 2)


def warmup_launches(warmup_ms, flops):
    """Launches that keep the device busy for about warmup_ms (priced at 1000 TFLOP/s, at least 10 us per launch)."""
    per_launch_ms = max(flops / 1.0e15 * 1e3, 0.010)
    return max(3, int(warmup_ms / per_launch_ms + 0.5))


def cmd_run(args):
    import numpy as np
    import torch

    import paper_2508_20258_amd as swz
    a, b = _inputs(args.workload)
    c = torch.empty((a.shape[0], b.shape[1]), dtype=torch.bfloat16, device="cuda")
    params = {}
    if args.tile:
        params.update(bm=args.tile, bn=args.tile)
    if args.group_m:
        params.update(group_m=args.group_m)
    if args.persistent:
        params.update(persistent=1)
    mode = swz.MODES[args.mode]
    warm = warmup_launches(args.warmup_ms, 2.0 * a.shape[0] * a.shape[1] * b.shape[1])
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(warm):                           # untimed; no synchronisation between these and the timed launches
        swz.gemm(a, b, c, mode=mode, **params)
    e0.record()
    for _ in range(args.launches):
        swz.gemm(a, b, c, mode=mode, **params)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / args.launches
    print(f"ran {warm} warm-up + {args.launches} timed launches of {args.workload} mode {args.mode}: {us:.2f} us per launch", flush=True)
    if args.check:
        # remap purity: the bits must equal those of the round-robin launch; the map must be a permutation
        ref = torch.empty_like(c)
        swz.gemm(a, b, ref, mode=swz.MODE_RR, **{k: v for k, v in params.items() if k != "persistent"})
        torch.cuda.synchronize()
        plan = swz.gemm_plan(a.shape[0], b.shape[1], a.shape[1], **params)
        m = swz.pid_map(plan["grid_m"], plan["grid_n"], plan["num_xcd"], plan["group_m"], mode)
        perm_ok = bool((np.sort(m) == np.arange(m.size)).all())
        same = bool(torch.equal(c.view(torch.int16), ref.view(torch.int16)))
        print(f"check: bit_identical_to_rr={same} map_is_permutation={perm_ok} us_per_launch={us:.3f}", flush=True)


# ---------------------------------------------------------------------------- candidate ranking

def parse_check_line(stdout):
    """(valid, us per launch) from the output of `run --check`; a run that printed no check line is invalid."""
    line = next((l for l in stdout.splitlines() if l.startswith("check:")), "")
    valid = "bit_identical_to_rr=True" in line and "map_is_permutation=True" in line
    try:
        us = float(line.split("us_per_launch=")[1].split()[0])
    except (IndexError, ValueError):
        us = float("nan")
    return valid, us


DEFAULT_CANDIDATE = ("xcd_groupm", 4, 256)          # what swz_gemm does when nothing is asked for
TIE_POINTS = 0.5                                    # measured hit rates closer than this are a tie


def rank_candidates(rows, tie_points=TIE_POINTS):
    """Order measured candidates of ONE tile shape and pick the best validated one.

    rows: dicts with mode, group_m, tile, valid, l2_hit_pct (measured), model_hit_pct, model_panels, us_per_launch.
    Broken candidates (valid false) and candidates without a measured hit rate are dropped.  The rest is
    ordered by measured L2 hit rate, highest first.  Candidates within `tie_points` of the best one are tied;
    among those the panel model decides (fewest distinct panels, i.e. least fabric traffic predicted), then the
    library default wins over anything else, then the simpler mapping (no renumbering, no grouping); timings of
    a few launches are printed but never break a tie.  Returns (ordered rows, best row or None, rows tied with it)."""
    good = [r for r in rows if r.get("valid") and r.get("l2_hit_pct") == r.get("l2_hit_pct") and r.get("l2_hit_pct") is not None]
    good.sort(key=lambda r: -r["l2_hit_pct"])
    if not good:
        return [], None, []
    simplicity = {"rr": 0, "groupm": 1, "xcd": 2, "xcd_groupm": 3}
    top = good[0]["l2_hit_pct"]
    tied = [r for r in good if top - r["l2_hit_pct"] <= tie_points]

    def key(r):
        is_default = (r["mode"], r.get("group_m") or 4) == DEFAULT_CANDIDATE[:2]
        return (r.get("model_panels", 0), 0 if is_default else 1, simplicity.get(r["mode"], 9), r.get("group_m") or 0)
    tied.sort(key=key)
    best = tied[0]
    return good, best, [r for r in tied if r is not best]


def pick_across_tiles(winners):
    """The winner among the per-tile-shape winners.  A hit rate is a ratio of requests, and a smaller tile asks the
    L2 for more lines per flop, so rates of different tile shapes do not compare; what they stand for does: the bytes
    that missed (TCC_MISS lines of 128 bytes), i.e. what crossed the fabric.  Fewest missed bytes wins; without that
    figure, the fewest predicted panel bytes."""
    winners = [w for w in winners if w is not None]
    if not winners:
        return None
    if all(w.get("l2_miss_mib") is not None for w in winners):
        return min(winners, key=lambda w: w["l2_miss_mib"])
    return min(winners, key=lambda w: w.get("model_panels", 0))


def candidate_list(group_ms, tiles):
    cands = []
    for tile in tiles:
        cands += [("rr", 0, tile), ("xcd", 0, tile)]
        cands += [(m, g, tile) for m in ("xcd_groupm", "groupm") for g in group_ms]
    return cands


def cmd_rank(args):
    """Profile candidate remaps in child processes and rank them by measured L2 hit rate."""
    import json
    import shutil
    import subprocess
    import tempfile

    import seeded_inputs as si

    import paper_2508_20258_amd as swz
    env = dict(os.environ, TMPDIR=os.environ.get("TMPDIR", "/tmp"))
    root = os.path.dirname(HERE)
    cfg = si.CONFIGS[args.workload]
    M, N, K = cfg["M"], cfg["N"], cfg["K"]
    X = args.num_xcd
    me = [sys.executable, "-m", "paper_2508_20258_amd.harness", "run", "--workload", args.workload]
    # 1. predict: the panel-count model on the library's own map, for every candidate (no GPU involved)
    rows = []
    for mode, g, tile in candidate_list(args.group_m, args.tile):
        plan = swz.gemm_plan(M, N, K, bm=tile, bn=tile, group_m=g or 4, num_xcd=X)
        m = swz.pid_map(plan["grid_m"], plan["grid_n"], X, plan["group_m"], swz.MODES[mode])
        hit, panels, _ = panel_model(m, plan["grid_n"], X, co_resident_tiles_per_xcd(tile, args.compute_units, X))
        rows.append(dict(mode=mode, group_m=g or None, tile=tile, model_hit_pct=100.0 * hit,
                         model_panels=panels * tile, valid=None, l2_hit_pct=None, us_per_launch=None))
    # 2. measure, most promising first; within a tile shape, candidates the model puts far below that shape's best are
    #    skipped (never the round-robin one: it is the baseline every candidate is validated against)
    rows.sort(key=lambda r: (-r["tile"], -r["model_hit_pct"]))
    best_model = {t: max(r["model_hit_pct"] for r in rows if r["tile"] == t) for t in args.tile}
    for r in rows:
        if r["mode"] != "rr" and best_model[r["tile"]] - r["model_hit_pct"] > args.prune_points:
            print(f"candidate {r['mode']:11s} group_m={r['group_m'] or '-':>2} tile {r['tile']}: model {r['model_hit_pct']:5.1f} %  skipped "
                  f"(more than {args.prune_points:g} points under the best prediction for this tile shape)", flush=True)
            continue
        extra = ["--mode", r["mode"], "--tile", str(r["tile"])] + (["--group-m", str(r["group_m"])] if r["group_m"] else [])
        chk = subprocess.run(me + extra + ["--check", "--warmup-ms", "40", "--launches", "20"], cwd=root, env=env, capture_output=True, text=True, timeout=600)
        r["valid"], r["us_per_launch"] = parse_check_line(chk.stdout)
        out = tempfile.mkdtemp(prefix="swz_rank_")
        try:
            prof = subprocess.run(["rocprofv3", "--pmc", "TCC_HIT", "TCC_MISS", "--output-format", "json", "-d", out, "--"]
                                  + me + extra + ["--warmup-ms", "0", "--launches", "2"],
                                  cwd=root, env=env, capture_output=True, text=True, timeout=600)
            if prof.returncode == 0:
                for d in summarize_json(out, "gemm").values():
                    h, m = d["counters"]["TCC_HIT"]["total"], d["counters"]["TCC_MISS"]["total"]
                    r["l2_hit_pct"] = 100.0 * h / (h + m)
                    r["l2_miss_mib"] = m * 128 / 2 ** 20
        finally:
            shutil.rmtree(out, ignore_errors=True)
        hit = r["l2_hit_pct"] if r["l2_hit_pct"] is not None else float("nan")
        print(f"candidate {r['mode']:11s} group_m={r['group_m'] or '-':>2} tile {r['tile']}: valid={r['valid']}  model {r['model_hit_pct']:5.1f} %  "
              f"measured L2 hit {hit:6.2f} %  missed {r.get('l2_miss_mib', float('nan')):8.1f} MiB  {r['us_per_launch']:9.2f} us", flush=True)
    measured = [r for r in rows if r["valid"] is not None]
    for r in measured:
        if not r["valid"]:
            print(f"dropped (broken remap): {r['mode']} group_m={r['group_m']} tile {r['tile']}")
    winners = []
    for tile in args.tile:
        good, best, tied = rank_candidates([r for r in measured if r["tile"] == tile])
        print(f"tile {tile}: ranking by measured L2 hit rate (within {TIE_POINTS} points = tie; ties broken by the panel model, then library default, then simplicity):")
        for r in good:
            print(f"  {r['mode']:11s} group_m={r['group_m'] or '-':>2}  measured {r['l2_hit_pct']:6.2f} %  model {r['model_hit_pct']:5.1f} %  "
                  f"missed {r.get('l2_miss_mib', float('nan')):8.1f} MiB  {r['us_per_launch']:9.2f} us")
        if best:
            print(f"  best of tile {tile}: {best['mode']} group_m={best['group_m']}"
                  + (" (tied with: " + ", ".join(f"{r['mode']}/g{r['group_m'] or '-'}" for r in tied) + ")" if tied else ""))
        winners.append(best)
    best = pick_across_tiles(winners)
    if best:
        print("best validated candidate (across tile shapes: fewest bytes missed in L2): " + json.dumps(best))
        good = [r for r in measured if r["valid"]]
        fastest = min(good, key=lambda r: r["us_per_launch"])
        print(f"fastest candidate (event timing of 20 launches, for information): {fastest['mode']} group_m={fastest['group_m']} tile {fastest['tile']} "
              f"{fastest['us_per_launch']:.2f} us")


# ---------------------------------------------------------------------------- full profile of one workload

PROFILE_MODES = ("rr", "xcd", "xcd_groupm")
SQ_COUNTERS = ["SQ_VALU_MFMA_BUSY_CYCLES", "SQ_INSTS_VALU_MFMA_MOPS_BF16", "SQ_LDS_BANK_CONFLICT", "SQ_LDS_IDX_ACTIVE",
               "SQ_BUSY_CU_CYCLES", "SQ_WAVE_CYCLES", "GRBM_GUI_ACTIVE"]
RECORD_PATH = os.path.join(HERE, "measured_counters.json")


def _one(directory, kernel, last=0):
    r = summarize(directory, kernel, last)
    return next(iter(r.values())) if r else None


def profile_table(src, workload, warmup_ms, launches, num_xcd=8, compute_units=256):
    """Text table and counter record from the rocprofv3 output directories `profile` wrote under src."""
    import seeded_inputs as si

    import paper_2508_20258_amd as swz
    cfg = si.CONFIGS[workload]
    M, N, K = cfg["M"], cfg["N"], cfg["K"]
    bm = cfg["tile"][0]
    gm, gn = -(-M // bm), -(-N // bm)
    flops = 2.0 * M * N * K
    copy_f = _one(f"{src}/copy_fetch", "copy")["counters"]["FETCH_SIZE"]
    copy_w = _one(f"{src}/copy_write", "copy")["counters"]["WRITE_SIZE"]
    fs, ws = 1024 * 1024 / copy_f, 1024 * 1024 / copy_w
    H = "python3 -m paper_2508_20258_amd.harness"
    run = f"{H} run --workload {workload} --mode MODE"
    lines = [f"rocprofv3 summary: swz gemm_bf16_kernel, workload {workload} (M={M} N={N} K={K}, tile {bm}x{bm}x64, grid {gm}x{gn}, {num_xcd} XCDs, group_m 4)",
             "MI355X (gfx950), one GPU.  Written by (repository root, TMPDIR=/tmp):",
             f"  {H} profile --workload {workload} --out <dir>",
             "which runs, for MODE in rr, xcd, xcd_groupm:",
             f"  rocprofv3 --kernel-trace --stats --output-format csv -d <out> -- {run} --warmup-ms {warmup_ms:g} --launches {launches}",
             f"  rocprofv3 --pmc TCC_HIT TCC_MISS --output-format json -d <out> -- {run} --warmup-ms 0 --launches 3",
             f"  rocprofv3 --pmc FETCH_SIZE --output-format csv -d <out> -- {run} --warmup-ms 0 --launches 3     (then the same with WRITE_SIZE)",
             f"  rocprofv3 --pmc {' '.join(SQ_COUNTERS)} --output-format csv -d <out> -- {run} --warmup-ms 0 --launches 3",
             f"  rocprofv3 --pmc FETCH_SIZE --output-format csv -d <out> -- {H} copy --mib 1024 --launches 3     (calibration; then WRITE_SIZE)",
             f"Byte-counter calibration on the plain 1 GiB copy kernel: FETCH_SIZE read {copy_f:.0f} KiB, WRITE_SIZE read {copy_w:.0f} KiB for 1048576 KiB",
             f"  => scale FETCH_SIZE by {fs:.3f}, WRITE_SIZE by {ws:.3f}.  Algorithmic minimum HBM bytes 2(MK+KN+MN) = {2 * (M * K + K * N + M * N) / 2 ** 20:.1f} MiB.",
             "L2 hit = TCC_HIT/(TCC_HIT+TCC_MISS) over all TCC instances; per XCD = the instances of each DIMENSION_XCC.",
             f"model = lock-step panel-count prediction on swz_pid_map's output, {co_resident_tiles_per_xcd(bm, compute_units, num_xcd)} co-resident tiles per XCD.",
             f"us = average kernel duration in the kernel trace over the last {launches} dispatches (the timed launches; the warm-up launches before them, {warmup_ms:g} ms of GPU time, are not averaged);",
             "first us = the same over the first 10 dispatches of the run (device idle before: boost clocks); worst us = the slowest dispatch of the run (the power controller's",
             "throttling a few milliseconds in).  event us = the run's own event timing per timed launch (includes launch gaps).", ""]
    lines.append(f"{'mode':11s} {'us':>9s} {'first us':>9s} {'worst us':>9s} {'event us':>9s} {'TFLOP/s':>8s} {'%peak':>6s} {'L2 hit%':>8s} {'model%':>7s} {'fetch MiB':>10s} {'write MiB':>10s} "
                 f"{'MfmaUtil%':>9s} {'LDS confl%':>10s}  per-XCD L2 hit %")
    record = {}
    for mode in PROFILE_MODES:
        t = f"{src}/{workload}_{mode}"
        kt = _one(f"{t}_kt", "gemm", launches)
        us = kt["warm_avg_ns"] / 1e3
        spans = sorted(summarize_spans(f"{t}_kt", "gemm"))
        cold = sum(d for _, d in spans[:10]) / max(len(spans[:10]), 1) / 1e3
        worst = max(d for _, d in spans) / 1e3
        ev = float("nan")
        try:
            with open(f"{t}_kt.log") as f:
                for l in f:
                    if "us per launch" in l:
                        ev = float(l.split(":")[-1].split("us per launch")[0])
        except OSError:
            pass
        tf = flops / (us * 1e-6) / 1e12
        tj = next(iter(summarize_json(f"{t}_tcc", "gemm").values()))["counters"]
        h, m = tj["TCC_HIT"], tj["TCC_MISS"]
        hit = 100 * h["total"] / (h["total"] + m["total"])
        per = [100 * a / (a + b) for a, b in zip(h["per_xcc"], m["per_xcc"])] if h["per_xcc"] else []
        fkib = _one(f"{t}_fetch", "gemm")["counters"]["FETCH_SIZE"] * fs
        wkib = _one(f"{t}_write", "gemm")["counters"]["WRITE_SIZE"] * ws
        sq = _one(f"{t}_sq", "gemm")["counters"]
        util = 100 * sq["SQ_VALU_MFMA_BUSY_CYCLES"] / (sq["GRBM_GUI_ACTIVE"] / num_xcd * compute_units * 4)
        confl = 100 * sq["SQ_LDS_BANK_CONFLICT"] / sq["SQ_LDS_IDX_ACTIVE"]
        tile_map = swz.pid_map(gm, gn, num_xcd, 4, swz.MODES[mode])
        model = 100 * panel_model(tile_map, gn, num_xcd, co_resident_tiles_per_xcd(bm, compute_units, num_xcd))[0]
        lines.append(f"{mode:11s} {us:9.2f} {cold:9.2f} {worst:9.2f} {ev:9.2f} {tf:8.1f} {tf / 25:6.1f} {hit:8.2f} {model:7.1f} {fkib / 1024:10.1f} {wkib / 1024:10.1f} "
                     f"{util:9.1f} {confl:10.2f}  " + " ".join(f"{r:.1f}" for r in per))
        record[mode] = dict(kernel_us=us, l2_hit_pct=hit, l2_hit_pct_per_xcd=per, model_hit_pct=model, fetch_bytes=int(fkib * 1024),
                            write_bytes=int(wkib * 1024), mfma_util_pct=util,
                            mfma_flop_issued=sq["SQ_INSTS_VALU_MFMA_MOPS_BF16"] * 512)
    issued = record["xcd_groupm"]["mfma_flop_issued"]
    lines += ["", f"MfmaUtil = SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE per XCD x {compute_units * 4} SIMDs).  MFMA flops cross-check: "
              f"SQ_INSTS_VALU_MFMA_MOPS_BF16 x 512 = {issued / 1e9:.1f} GFLOP issued vs 2MNK = {flops / 1e9:.1f} GFLOP (edge tiles compute padding)."]
    return "\n".join(lines) + "\n", record


def summarize_spans(directory, kernel_filter):
    """(start, duration) in ns of every dispatch whose kernel name contains kernel_filter."""
    out = []
    for path in glob.glob(os.path.join(directory, "**", "*kernel_trace.csv"), recursive=True):
        for r in _rows(path):
            if kernel_filter in r["Kernel_Name"]:
                out.append((int(r["Start_Timestamp"]), int(r["End_Timestamp"]) - int(r["Start_Timestamp"])))
    return out


def _rocprof(out, tag, fmt, prof_args, prog_args, limit=180):
    """One rocprofv3 run of `python -m paper_2508_20258_amd.harness <prog_args>` into <out>/<tag> (log beside it)."""
    import shutil
    import subprocess
    env = dict(os.environ, TMPDIR=os.environ.get("TMPDIR", "/tmp"))
    d = os.path.join(out, tag)
    shutil.rmtree(d, ignore_errors=True)          # a pass directory holds one run: the readers sum over every file they find
    res = subprocess.run(["rocprofv3", *prof_args, "--output-format", fmt, "-d", d, "--", sys.executable, "-m",
                          "paper_2508_20258_amd.harness", *prog_args],
                         cwd=os.path.dirname(HERE), env=env, capture_output=True, text=True, timeout=limit)
    with open(d + ".log", "w") as f:
        f.write(res.stdout + res.stderr)
    if res.returncode != 0:
        sys.exit(f"rocprofv3 pass {tag} failed ({res.returncode}):\n{(res.stdout + res.stderr)[-2000:]}")
    print(f"pass {tag} done", flush=True)


def cmd_profile_transpose(args):
    """rocprofv3 passes for swz_transpose over tile x mapping, as child processes; prints the summary table."""
    out = os.path.abspath(args.out)
    os.makedirs(out, exist_ok=True)
    m, n = args.m, args.n
    base = ["transpose", "--m", str(m), "--n", str(n)]
    combos = [(t, mo) for t in args.tile for mo in args.mode]
    if not args.table_only:
        for c, tag in (("FETCH_SIZE", "copy_fetch"), ("WRITE_SIZE", "copy_write")):
            _rocprof(out, tag, "csv", ["--pmc", c], ["copy", "--mib", "1024", "--launches", "3"])
        _rocprof(out, "copy_kt", "csv", ["--kernel-trace", "--stats"], ["copy", "--mib", str(4 * m * n >> 21), "--launches", str(args.launches + 1)])
        for tile, mode in combos:
            prog = base + ["--tile", str(tile), "--mode", mode]
            t = f"t{tile}_{mode}"
            _rocprof(out, t + "_kt", "csv", ["--kernel-trace", "--stats"], prog + ["--launches", str(args.launches + 1)])
            _rocprof(out, t + "_tcc", "json", ["--pmc", "TCC_HIT", "TCC_MISS"], prog + ["--launches", "3"])
            _rocprof(out, t + "_fetch", "csv", ["--pmc", "FETCH_SIZE"], prog + ["--launches", "3"])
            _rocprof(out, t + "_write", "csv", ["--pmc", "WRITE_SIZE"], prog + ["--launches", "3"])
    fs = 1024 * 1024 / _one(f"{out}/copy_fetch", "copy")["counters"]["FETCH_SIZE"]
    ws = 1024 * 1024 / _one(f"{out}/copy_write", "copy")["counters"]["WRITE_SIZE"]
    copy_us = _one(f"{out}/copy_kt", "copy", args.launches)["warm_avg_ns"] / 1e3
    copy_gbs = 4.0 * m * n / (copy_us * 1e-6) / 1e9
    H = "python3 -m paper_2508_20258_amd.harness"
    lines = [f"rocprofv3 summary: swz transpose16_kernel, {m} x {n} 16-bit elements ({2 * m * n >> 20} MiB in, {2 * m * n >> 20} MiB out), MI355X, one GPU.",
             "Written by (repository root, TMPDIR=/tmp):",
             f"  {H} profile-transpose --m {m} --n {n} --out <dir>",
             f"which runs, for TILE in {', '.join(map(str, args.tile))} and MODE in {', '.join(args.mode)}:",
             f"  rocprofv3 --kernel-trace --stats --output-format csv -d <out> -- {H} transpose --m {m} --n {n} --tile TILE --mode MODE --launches {args.launches + 1}",
             f"  rocprofv3 --pmc TCC_HIT TCC_MISS --output-format json -d <out> -- {H} transpose --m {m} --n {n} --tile TILE --mode MODE --launches 3",
             "  rocprofv3 --pmc FETCH_SIZE (then WRITE_SIZE) --output-format csv -d <out> -- the same",
             f"  and the same passes on `{H} copy` (byte-counter calibration on 1 GiB: FETCH_SIZE x {fs:.3f}, WRITE_SIZE x {ws:.3f}; kernel trace on {4 * m * n >> 20} MiB moved).",
             f"Roofline: HBM, 8 TB/s; algorithmic bytes 4*M*N = {4 * m * n >> 20} MiB per launch.  us = kernel duration in the kernel trace, average over the last {args.launches} launches.",
             f"The library's plain copy kernel on the same amount of data in the same session: {copy_us:.2f} us = {copy_gbs:.0f} GB/s ({100 * copy_gbs / 8000:.1f} % of 8 TB/s).",
             "", f"{'tile':>4s} {'mode':16s} {'us':>8s} {'GB/s':>6s} {'% of 8 TB/s':>11s} {'x copy':>7s} {'L2 hit %':>8s} {'fetch MiB':>10s} {'write MiB':>10s}"]
    for tile, mode in combos:
        t = f"{out}/t{tile}_{mode}"
        us = _one(t + "_kt", "transpose", args.launches)["warm_avg_ns"] / 1e3
        gbs = 4.0 * m * n / (us * 1e-6) / 1e9
        tj = next(iter(summarize_json(t + "_tcc", "transpose").values()))["counters"]
        hit = 100 * tj["TCC_HIT"]["total"] / (tj["TCC_HIT"]["total"] + tj["TCC_MISS"]["total"])
        f = _one(t + "_fetch", "transpose")["counters"]["FETCH_SIZE"] * fs / 1024
        w = _one(t + "_write", "transpose")["counters"]["WRITE_SIZE"] * ws / 1024
        lines.append(f"{tile:4d} {mode:16s} {us:8.2f} {gbs:6.0f} {100 * gbs / 8000:11.1f} {gbs / copy_gbs:7.2f} {hit:8.2f} {f:10.1f} {w:10.1f}")
    text = "\n".join(lines) + "\n"
    print(text, flush=True)
    with open(os.path.join(out, f"transpose_{m}x{n}.txt"), "w") as f:
        f.write(text)


ROW_CASES = [  # (M, N, chunks, mode): chunked rows under both dispatch orders, one workgroup per row, one wave per row, beyond the cache
    (1024, 65536, 8, "rr"), (1024, 65536, 8, "xcd"), (1024, 65536, 1, "rr"), (8192, 8192, 8, "rr"), (8192, 8192, 8, "xcd"),
    (8192, 8192, 1, "rr"), (65536, 1024, 1, "rr"), (32768, 16384, 1, "rr")]


def cmd_profile_rows(args):
    """rocprofv3 passes for swz_softmax / swz_layernorm over ROW_CASES, as child processes; prints the summary table."""
    out = os.path.abspath(args.out)
    os.makedirs(out, exist_ok=True)
    cases = [(op, m, n, c, mode) for op in ("softmax", "layernorm") for (m, n, c, mode) in ROW_CASES]
    if not args.table_only:
        for c, tag in (("FETCH_SIZE", "copy_fetch"), ("WRITE_SIZE", "copy_write")):
            _rocprof(out, tag, "csv", ["--pmc", c], ["copy", "--mib", "1024", "--launches", "3"])
        _rocprof(out, "copy_kt", "csv", ["--kernel-trace", "--stats"], ["copy", "--mib", "1024", "--launches", str(args.launches + 1)])
        for op, m, n, c, mode in cases:
            prog = ["rows", "--op", op, "--m", str(m), "--n", str(n), "--chunks", str(c), "--mode", mode]
            t = f"{op}_{m}x{n}_c{c}_{mode}"
            _rocprof(out, t + "_kt", "csv", ["--kernel-trace", "--stats"], prog + ["--launches", str(args.launches + 1)])
            _rocprof(out, t + "_tcc", "json", ["--pmc", "TCC_HIT", "TCC_MISS"], prog + ["--launches", "3"])
            _rocprof(out, t + "_fetch", "csv", ["--pmc", "FETCH_SIZE"], prog + ["--launches", "3"])
            _rocprof(out, t + "_write", "csv", ["--pmc", "WRITE_SIZE"], prog + ["--launches", "3"])
    fs = 1024 * 1024 / _one(f"{out}/copy_fetch", "copy")["counters"]["FETCH_SIZE"]
    ws = 1024 * 1024 / _one(f"{out}/copy_write", "copy")["counters"]["WRITE_SIZE"]
    copy_us = _one(f"{out}/copy_kt", "copy", args.launches)["warm_avg_ns"] / 1e3
    copy_gbs = 2.0 * (1 << 30) / (copy_us * 1e-6) / 1e9
    H = "python3 -m paper_2508_20258_amd.harness"
    lines = ["rocprofv3 summary: swz softmax_rows_kernel / layernorm_rows_kernel, bf16, MI355X, one GPU.",
             "Written by (repository root, TMPDIR=/tmp):",
             f"  {H} profile-rows --out <dir>",
             "which runs, for OP in softmax, layernorm and (M, N, CHUNKS, MODE) as in the table:",
             f"  rocprofv3 --kernel-trace --stats --output-format csv -d <out> -- {H} rows --op OP --m M --n N --chunks CHUNKS --mode MODE --launches {args.launches + 1}",
             f"  rocprofv3 --pmc TCC_HIT TCC_MISS --output-format json -d <out> -- {H} rows --op OP --m M --n N --chunks CHUNKS --mode MODE --launches 3",
             "  rocprofv3 --pmc FETCH_SIZE (then WRITE_SIZE) --output-format csv -d <out> -- the same",
             f"  and the same passes on `{H} copy --mib 1024` (byte-counter calibration: FETCH_SIZE x {fs:.3f}, WRITE_SIZE x {ws:.3f}).",
             "Roofline: HBM, 8 TB/s; algorithmic bytes 4*M*N per launch (read x once, write y once): 256 MiB, 2 GiB for 32768 x 16384.",
             "Launches repeat over the same data; 256 MiB is partly held by the 256 MB memory-side cache between launches, 2 GiB is not.",
             f"The library's plain copy kernel, 1 GiB in + 1 GiB out, same session: {copy_us:.2f} us = {copy_gbs:.0f} GB/s ({100 * copy_gbs / 8000:.1f} % of 8 TB/s).",
             f"us = kernel duration in the kernel trace, average over the last {args.launches} launches.  chunks = workgroups per row; each reads the whole row.",
             "", f"{'op':9s} {'M x N':>14s} {'chunks':>6s} {'mode':5s} {'us':>8s} {'GB/s':>6s} {'% of 8 TB/s':>11s} {'L2 hit %':>8s} {'fetch MiB':>10s} {'write MiB':>10s}"]
    for op, m, n, c, mode in cases:
        t = f"{out}/{op}_{m}x{n}_c{c}_{mode}"
        us = _one(t + "_kt", "rows_kernel", args.launches)["warm_avg_ns"] / 1e3
        gbs = 4.0 * m * n / (us * 1e-6) / 1e9
        tj = next(iter(summarize_json(t + "_tcc", "rows_kernel").values()))["counters"]
        hit = 100 * tj["TCC_HIT"]["total"] / (tj["TCC_HIT"]["total"] + tj["TCC_MISS"]["total"])
        f = _one(t + "_fetch", "rows_kernel")["counters"]["FETCH_SIZE"] * fs / 1024
        w = _one(t + "_write", "rows_kernel")["counters"]["WRITE_SIZE"] * ws / 1024
        lines.append(f"{op:9s} {m:>6d} x {n:<6d} {c:6d} {mode:5s} {us:8.2f} {gbs:6.0f} {100 * gbs / 8000:11.1f} {hit:8.2f} {f:10.1f} {w:10.1f}")
    text = "\n".join(lines) + "\n"
    print(text, flush=True)
    with open(os.path.join(out, "rowwise_softmax_layernorm.txt"), "w") as f:
        f.write(text)


def cmd_profile(args):
    """Every rocprofv3 pass for the three mappings of one workload, as child processes; prints the summary table."""
    import json
    out = os.path.abspath(args.out)
    os.makedirs(out, exist_ok=True)

    def rocprof(tag, fmt, prof_args, prog_args):
        _rocprof(out, tag, fmt, prof_args, prog_args)

    if not args.table_only:
        for c, tag in (("FETCH_SIZE", "copy_fetch"), ("WRITE_SIZE", "copy_write")):
            rocprof(tag, "csv", ["--pmc", c], ["copy", "--mib", "1024", "--launches", "3"])
        for mode in PROFILE_MODES:
            run = ["run", "--workload", args.workload, "--mode", mode]
            short = run + ["--warmup-ms", "0", "--launches", "3"]
            t = f"{args.workload}_{mode}"
            rocprof(t + "_kt", "csv", ["--kernel-trace", "--stats"], run + ["--warmup-ms", str(args.warmup_ms), "--launches", str(args.launches)])
            rocprof(t + "_tcc", "json", ["--pmc", "TCC_HIT", "TCC_MISS"], short)
            rocprof(t + "_fetch", "csv", ["--pmc", "FETCH_SIZE"], short)
            rocprof(t + "_write", "csv", ["--pmc", "WRITE_SIZE"], short)
            rocprof(t + "_sq", "csv", ["--pmc", *SQ_COUNTERS], short)
    text, record = profile_table(out, args.workload, args.warmup_ms, args.launches)
    print(text, flush=True)
    with open(os.path.join(out, f"gemm_{args.workload}.txt"), "w") as f:
        f.write(text)
    if args.record:
        doc = {"kernel_sha256": kernel_hash(), "workloads": {}}
        if os.path.exists(RECORD_PATH):
            with open(RECORD_PATH) as f:
                old = json.load(f)
            if old.get("kernel_sha256") == doc["kernel_sha256"]:
                doc = old
        doc["workloads"][args.workload] = record
        with open(RECORD_PATH, "w") as f:
            json.dump(doc, f, indent=1, sort_keys=True)
            f.write("\n")
        print(f"recorded counters of {args.workload} in {RECORD_PATH}", flush=True)


def recorded_counters(workload=None):
    """Counters `profile --record` stored for the kernel sources as they are now; None when the sources have changed."""
    import json
    try:
        with open(RECORD_PATH) as f:
            doc = json.load(f)
    except OSError:
        return None
    if doc.get("kernel_sha256") != kernel_hash():
        return None
    return doc["workloads"] if workload is None else doc["workloads"].get(workload)


# ---------------------------------------------------------------------------- what bounds the kernel: clocks per XCD

def clocks_report(probe, flops, label):
    """Text report from the stamps of one swz_gemm_probe launch (probe: int array, workgroups x 16, see include/swz.h).

    The shader clock counter advances with the compute clock of the XCD the workgroup runs on, the other counter
    at a constant 100 MHz, so their ratio over the K loop is the clock the XCD sustained under the kernel."""
    import numpy as np
    p = np.asarray(probe, dtype=np.int64)
    xcc = p[:, 8]
    steps = p[0, 10]
    t0 = p[:, 1].min()                                     # first workgroup entry, 100 MHz ticks
    loop_cyc = (p[:, 4] - p[:, 2]).astype(np.float64)
    loop_us = (p[:, 5] - p[:, 3]) / 100.0
    mhz = loop_cyc / np.maximum(loop_us, 1e-9)
    lines = [label,
             f"workgroups {p.shape[0]}, K steps of 32 per tile {steps}; a K step of a 256x256 tile is 1024 clocks of MFMA issue per SIMD "
             f"(512 for a 128x128 tile)",
             f"{'XCD':>3s} {'tiles':>5s} {'cyc/step':>9s} {'min':>7s} {'max':>7s} {'MHz in loop':>11s} {'min':>6s} {'max':>6s} "
             f"{'open us':>8s} {'loop us':>8s} {'store us':>8s} {'first end us':>12s} {'last end us':>11s}"]
    for x in sorted(set(xcc.tolist())):
        s = xcc == x
        cps = loop_cyc[s] / steps
        open_us = ((p[s, 3] - p[s, 1]) / 100.0).mean()
        store_us = ((p[s, 7] - p[s, 5]) / 100.0).mean()
        ends = (p[s, 7] - t0) / 100.0
        lines.append(f"{x:3d} {int(s.sum()):5d} {cps.mean():9.1f} {cps.min():7.1f} {cps.max():7.1f} {mhz[s].mean():11.0f} {mhz[s].min():6.0f} "
                     f"{mhz[s].max():6.0f} {open_us:8.2f} {loop_us[s].mean():8.2f} {store_us:8.2f} {ends.min():12.2f} {ends.max():11.2f}")
    span_us = (p[:, 7].max() - t0) / 100.0
    busy = loop_us.sum() / (p.shape[0] * span_us) if p.shape[0] <= 256 else float("nan")
    lines.append(f"all: {loop_cyc.mean() / steps:.1f} cycles per K step, {mhz.mean():.0f} MHz in the loop "
                 f"(slowest XCD {min(mhz[xcc == x].mean() for x in set(xcc.tolist())):.0f}, fastest "
                 f"{max(mhz[xcc == x].mean() for x in set(xcc.tolist())):.0f}); first entry to last store issued {span_us:.2f} us "
                 f"= {flops / span_us / 1e6:.0f} TFLOP/s" + (f"; the K loops fill {100 * busy:.1f} % of that span" if busy == busy else ""))
    return "\n".join(lines)


def cmd_clocks(args):
    import torch

    import paper_2508_20258_amd as swz
    a, b = _inputs(args.workload)
    c = torch.empty((a.shape[0], b.shape[1]), dtype=torch.bfloat16, device="cuda")
    mode = swz.MODES[args.mode]
    params = dict(bm=args.tile, bn=args.tile) if args.tile else {}
    flops = 2.0 * a.shape[0] * a.shape[1] * b.shape[1]
    _, probe = swz.gemm_probe(a, b, c, mode=mode, **params)          # loads the stamped kernel's code before the measurement
    torch.cuda.synchronize()
    warm = warmup_launches(args.warmup_ms, flops)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(warm):                                  # the product kernel; the stamped launch follows without a gap
        swz.gemm(a, b, c, mode=mode, **params)
    e0.record()
    swz.gemm_probe(a, b, c, mode=mode, probe=probe, **params)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3
    label = (f"swz_gemm_probe, workload {args.workload}, mode {args.mode}, launched right behind {warm} warm-up launches "
             f"({args.warmup_ms:g} ms) of the product kernel; the stamped launch took {us:.2f} us between events ({flops / us / 1e6:.0f} TFLOP/s)")
    print(clocks_report(probe.cpu().numpy(), flops, label), flush=True)


def cmd_transpose(args):
    import torch

    import paper_2508_20258_amd as swz
    torch.manual_seed(0)
    if args.elem_bytes == 4:
        x = torch.randint(-(1 << 31), (1 << 31) - 1, (args.m, args.n), dtype=torch.int32, device="cuda")
    else:
        x = torch.randint(-32768, 32767, (args.m, args.n), dtype=torch.int16, device="cuda").view(torch.bfloat16)
    out = torch.empty((args.n, args.m), dtype=x.dtype, device="cuda")
    mode = swz.MODES[args.mode]
    params = dict(group_m=args.group_m) if args.group_m else {}
    swz.transpose(x, out, tile=args.tile, mode=mode, **params)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(max(args.launches - 1, 1)):
        swz.transpose(x, out, tile=args.tile, mode=mode, **params)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / max(args.launches - 1, 1)
    gbs = 2.0 * args.elem_bytes * args.m * args.n / (us * 1e-6) / 1e9
    print(f"ran {args.launches} transposes {args.m}x{args.n} ({args.elem_bytes}-byte elements) tile {args.tile} mode {args.mode} group_m {args.group_m or 4}: {us:.2f} us per launch, "
          f"{gbs:.0f} GB/s of 2*M*N*elem_bytes bytes ({100 * gbs / 8000:.1f} % of 8 TB/s)", flush=True)


def cmd_rows(args):
    import torch

    import paper_2508_20258_amd as swz
    torch.manual_seed(0)
    x = (torch.randn((args.m, args.n), device="cuda") * 2.0).to(torch.bfloat16)
    out = torch.empty_like(x)
    g = torch.rand(args.n, device="cuda").to(torch.bfloat16)
    b = torch.rand(args.n, device="cuda").to(torch.bfloat16)
    mode = swz.MODES[args.mode]

    def launch():
        if args.op == "softmax":
            swz.softmax(x, out, chunks=args.chunks, mode=mode)
        else:
            swz.layernorm(x, g, b, out, eps=1e-5, chunks=args.chunks, mode=mode)

    launch()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(max(args.launches - 1, 1)):
        launch()
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / max(args.launches - 1, 1)
    gbs = 4.0 * args.m * args.n / (us * 1e-6) / 1e9
    print(f"ran {args.launches} x {args.op} {args.m}x{args.n} chunks {args.chunks} mode {args.mode}: {us:.2f} us per launch, "
          f"{gbs:.0f} GB/s of 4*M*N bytes ({100 * gbs / 8000:.1f} % of 8 TB/s)", flush=True)


def cmd_peak(args):
    """Data-sheet MFMA peak from the device's unit counts, and the rate the device sustains on register operands."""
    import torch

    import paper_2508_20258_amd as swz
    info = swz.device_info()
    cus = info["compute_units"]
    sheet = cus * 4 * 1024 * 2.4e9 / 1e12
    print(f"data sheet: {cus} CUs x 4 SIMDs x 1024 flop/clk (one 16x16x32 bf16 MFMA = 16384 flop per 16 clocks) x 2.4 GHz "
          f"= {sheet:.1f} TFLOP/s (published: 2.5 PFLOP/s dense bf16)")
    out = torch.empty(cus * 512, dtype=torch.float32, device="cuda")
    for name, rnd in (("zero operands", False), ("random bf16 operands", True)):
        swz.mfma_peak(out, 2000, rnd)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flop = swz.mfma_peak(out, args.iters, rnd)
        e1.record()
        torch.cuda.synchronize()
        t = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
        print(f"measured, {name}: {t:.1f} TFLOP/s = {100 * t / sheet:.1f} % of the data-sheet figure "
              f"(sustained clock ~{2.4 * t / sheet:.2f} GHz if every SIMD issues back to back)", flush=True)


def cmd_copy(args):
    import torch

    import paper_2508_20258_amd as swz
    n = args.mib << 20
    src = torch.ones(n, dtype=torch.uint8, device="cuda")
    dst = torch.zeros(n, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    for _ in range(args.launches):
        swz.copy_bytes(src, dst)
    torch.cuda.synchronize()
    print(f"ran {args.launches} copies of {args.mib} MiB (reads {n} B, writes {n} B each)", flush=True)


def _rows(path):
    with open(path, newline="") as f:
        yield from csv.DictReader(f)


def summarize(directory, kernel_filter=None, last=0):
    """Returns {kernel name: {"n": dispatches, "avg_ns": ..., "warm_avg_ns": ..., "counters": {name: avg per dispatch}}}.

    warm_avg_ns is the average over the last `last` dispatches in start order (the later half if `last` is 0): a run
    started on an idle device spends its first launches ramping the clock up, and `run` puts its untimed warm-up
    launches first."""
    out = defaultdict(lambda: {"n": 0, "total_ns": 0, "spans": [], "counters": defaultdict(float), "counter_n": defaultdict(int)})
    for path in glob.glob(os.path.join(directory, "**", "*kernel_trace.csv"), recursive=True):
        for r in _rows(path):
            k = r["Kernel_Name"]
            out[k]["n"] += 1
            out[k]["total_ns"] += int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
            out[k]["spans"].append((int(r["Start_Timestamp"]), int(r["End_Timestamp"]) - int(r["Start_Timestamp"])))
    for path in glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True):
        per_dispatch = defaultdict(float)
        for r in _rows(path):
            per_dispatch[(r["Kernel_Name"], r["Dispatch_Id"], r["Counter_Name"])] += float(r["Counter_Value"])
        for (k, _, cname), v in per_dispatch.items():
            out[k]["counters"][cname] += v
            out[k]["counter_n"][cname] += 1
    res = {}
    for k, d in out.items():
        if kernel_filter and kernel_filter not in k:
            continue
        durs = [dur for _, dur in sorted(d["spans"])]
        late = durs[-last:] if 0 < last <= len(durs) else durs[len(durs) // 2:]
        res[k] = {"n": d["n"], "avg_ns": d["total_ns"] / d["n"] if d["n"] else None,
                  "warm_avg_ns": sum(late) / len(late) if late else None,
                  "counters": {c: d["counters"][c] / d["counter_n"][c] for c in d["counters"]}}
    return res


def summarize_json(directory, kernel_filter=None):
    """Per-kernel, per-counter averages from rocprofv3 JSON output, split by XCC where a counter has that dimension.

    Returns {kernel: {"n": dispatches, "counters": {name: {"total": avg per dispatch, "per_xcc": [avg, ...] or None}}}}.
    A dispatch's records follow the order of the counter's `instances` list.
    """
    import json
    out = {}
    for path in glob.glob(os.path.join(directory, "**", "*results.json"), recursive=True):
        with open(path) as f:
            doc = json.load(f)
        for tool in doc["rocprofiler-sdk-tool"]:
            counters = {c["id"]["handle"]: c for c in tool["counters"]}
            names = {k["kernel_id"]: k.get("formatted_kernel_name") or k.get("kernel_name") for k in tool["kernel_symbols"]}
            for disp in tool["callback_records"].get("counter_collection", []):
                info = disp["dispatch_data"]["dispatch_info"]
                kname = names.get(info["kernel_id"], str(info["kernel_id"]))
                if kernel_filter and kernel_filter not in kname:
                    continue
                k = out.setdefault(kname, {"n": 0, "counters": {}})
                k["n"] += 1
                seen = defaultdict(int)
                for rec in disp["records"]:
                    c = counters[rec["counter_id"]["handle"]]
                    inst = c["instances"][seen[c["name"]]] if seen[c["name"]] < len(c["instances"]) else None
                    seen[c["name"]] += 1
                    slot = k["counters"].setdefault(c["name"], {"total": 0.0, "per_xcc": defaultdict(float)})
                    slot["total"] += rec["value"]
                    if inst is not None:
                        for dim in inst["dimensions"]:
                            if dim["dimension_name"] == "DIMENSION_XCC":
                                slot["per_xcc"][dim["index"]] += rec["value"]
    for k in out.values():
        for slot in k["counters"].values():
            slot["total"] /= k["n"]
            slot["per_xcc"] = [slot["per_xcc"][i] / k["n"] for i in sorted(slot["per_xcc"])] or None
    return out


def cmd_summarize(args):
    for kname, d in sorted(summarize_json(args.dir, args.kernel).items()):
        short = kname if len(kname) < 100 else kname[:97] + "..."
        print(f"kernel: {short}\n  dispatches with counters {d['n']}")
        c = d["counters"]
        for name in sorted(c):
            print(f"  {name:34s} {c[name]['total']:.6g}   (average per dispatch)")
        if "TCC_HIT" in c and "TCC_MISS" in c:
            h, m = c["TCC_HIT"], c["TCC_MISS"]
            print(f"  L2 hit rate = TCC_HIT/(TCC_HIT+TCC_MISS) = {100 * h['total'] / (h['total'] + m['total']):.2f} %")
            if h["per_xcc"] and m["per_xcc"]:
                rates = [100 * a / (a + b) if a + b else float('nan') for a, b in zip(h["per_xcc"], m["per_xcc"])]
                print("  per XCD: " + " ".join(f"{r:.2f}" for r in rates) + " %")
    res = summarize(args.dir, args.kernel)
    for k, d in sorted(res.items()):
        short = k if len(k) < 100 else k[:97] + "..."
        print(f"kernel: {short}")
        if d["n"]:
            print(f"  dispatches {d['n']}  avg duration {d['avg_ns'] / 1e3:.2f} us")
        c = d["counters"]
        for name in sorted(c):
            print(f"  {name:34s} {c[name]:.6g}   (average per dispatch)")
        if "TCC_HIT_sum" in c and "TCC_MISS_sum" in c and c["TCC_HIT_sum"] + c["TCC_MISS_sum"] > 0:
            print(f"  L2 hit rate = TCC_HIT/(TCC_HIT+TCC_MISS) = {100 * c['TCC_HIT_sum'] / (c['TCC_HIT_sum'] + c['TCC_MISS_sum']):.2f} %")


def main(argv=None):
    ap = argparse.ArgumentParser(prog="harness")
    sub = ap.add_subparsers(dest="cmd", required=True)
    r = sub.add_parser("run")
    r.add_argument("--workload", default="cfg2_4096")
    r.add_argument("--mode", default="xcd_groupm", choices=MODE_NAMES)
    r.add_argument("--launches", type=int, default=20, help="timed launches")
    r.add_argument("--warmup-ms", type=float, default=40.0, help="GPU time of untimed launches before the timed ones")
    r.add_argument("--tile", type=int, default=0)
    r.add_argument("--group-m", type=int, default=0)
    r.add_argument("--persistent", action="store_true")
    r.add_argument("--check", action="store_true", help="also compare the bits with a round-robin launch")
    r.set_defaults(fn=cmd_run)
    k = sub.add_parser("rank")
    k.add_argument("--workload", default="cfg4_skinny")
    k.add_argument("--group-m", type=int, nargs="+", default=[1, 2, 4, 8, 16])
    k.add_argument("--tile", type=int, nargs="+", default=[256, 128])
    k.add_argument("--num-xcd", type=int, default=8, help="XCDs of the device the children run on (the parent never touches it)")
    k.add_argument("--compute-units", type=int, default=256)
    k.add_argument("--prune-points", type=float, default=5.0, help="skip candidates the model puts this many points under its best")
    k.set_defaults(fn=cmd_rank)
    pf = sub.add_parser("profile")
    pf.add_argument("--workload", default="cfg2_4096")
    pf.add_argument("--out", required=True)
    pf.add_argument("--warmup-ms", type=float, default=40.0)
    pf.add_argument("--launches", type=int, default=20)
    pf.add_argument("--record", action="store_true", help="store the counters, keyed by the kernel source hash, for bench.py")
    pf.add_argument("--table-only", action="store_true", help="only rebuild the table from passes already under --out")
    pf.set_defaults(fn=cmd_profile)
    pt = sub.add_parser("profile-transpose")
    pt.add_argument("--m", type=int, default=16384)
    pt.add_argument("--n", type=int, default=16384)
    pt.add_argument("--out", required=True)
    pt.add_argument("--tile", type=int, nargs="+", default=[64, 128, 32])
    pt.add_argument("--mode", nargs="+", default=["rr", "xcd", "xcd_groupm", "rr_skew", "xcd_skew", "xcd_groupm_skew"], choices=MODE_NAMES)
    pt.add_argument("--launches", type=int, default=20)
    pt.add_argument("--table-only", action="store_true")
    pt.set_defaults(fn=cmd_profile_transpose)
    pr = sub.add_parser("profile-rows")
    pr.add_argument("--out", required=True)
    pr.add_argument("--launches", type=int, default=10)
    pr.add_argument("--table-only", action="store_true")
    pr.set_defaults(fn=cmd_profile_rows)
    ck = sub.add_parser("clocks")
    ck.add_argument("--workload", default="cfg2_4096")
    ck.add_argument("--mode", default="xcd_groupm", choices=MODE_NAMES)
    ck.add_argument("--tile", type=int, default=0)
    ck.add_argument("--warmup-ms", type=float, default=40.0)
    ck.set_defaults(fn=cmd_clocks)
    t = sub.add_parser("transpose")
    t.add_argument("--m", type=int, default=16384)
    t.add_argument("--n", type=int, default=16384)
    t.add_argument("--tile", type=int, default=64, choices=[32, 64, 128])
    t.add_argument("--elem-bytes", type=int, default=2, choices=[2, 4])
    t.add_argument("--mode", default="xcd_groupm_skew", choices=MODE_NAMES)
    t.add_argument("--launches", type=int, default=10)
    t.add_argument("--group-m", type=int, default=0)
    t.set_defaults(fn=cmd_transpose)
    w = sub.add_parser("rows")
    w.add_argument("--op", default="softmax", choices=["softmax", "layernorm"])
    w.add_argument("--m", type=int, default=8192)
    w.add_argument("--n", type=int, default=8192)
    w.add_argument("--chunks", type=int, default=8)
    w.add_argument("--mode", default="xcd", choices=MODE_NAMES)
    w.add_argument("--launches", type=int, default=10)
    w.set_defaults(fn=cmd_rows)
    pk = sub.add_parser("peak")
    pk.add_argument("--iters", type=int, default=20000)
    pk.set_defaults(fn=cmd_peak)
    c = sub.add_parser("copy")
    c.add_argument("--mib", type=int, default=1024)
    c.add_argument("--launches", type=int, default=3)
    c.set_defaults(fn=cmd_copy)
    s = sub.add_parser("summarize")
    s.add_argument("dir")
    s.add_argument("--kernel", default=None)
    s.set_defaults(fn=cmd_summarize)
    args = ap.parse_args(argv)
    args.fn(args)


if __name__ == "__main__":
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    main()
