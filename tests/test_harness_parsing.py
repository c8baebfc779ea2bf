"""The profiling harness's readers, on small hand-written files in rocprofv3's CSV / JSON layouts."""
import json
import os

from paper_2508_20258_amd import harness


def test_csv_summary(tmp_path):
    d = tmp_path / "run" / "host"
    os.makedirs(d)
    (d / "1_kernel_trace.csv").write_text(
        '"Kind","Kernel_Name","Start_Timestamp","End_Timestamp"\n'
        '"KERNEL_DISPATCH","gemm<2>",1000,3000\n"KERNEL_DISPATCH","gemm<2>",5000,6000\n"KERNEL_DISPATCH","copy",0,500\n')
    (d / "1_counter_collection.csv").write_text(
        '"Dispatch_Id","Kernel_Name","Counter_Name","Counter_Value"\n'
        '1,"gemm<2>","TCC_HIT_sum",30\n1,"gemm<2>","TCC_MISS_sum",10\n2,"gemm<2>","TCC_HIT_sum",50\n2,"gemm<2>","TCC_MISS_sum",10\n'
        '1,"gemm<2>","FETCH_SIZE",7.5\n1,"gemm<2>","FETCH_SIZE",2.5\n')          # two rows of one dispatch add up
    r = harness.summarize(str(tmp_path / "run"), "gemm")
    assert list(r) == ["gemm<2>"]
    g = r["gemm<2>"]
    assert g["n"] == 2 and g["avg_ns"] == 1500
    assert g["warm_avg_ns"] == 1000                             # the later half of the dispatches: the second one
    assert g["counters"]["TCC_HIT_sum"] == 40 and g["counters"]["TCC_MISS_sum"] == 10
    assert g["counters"]["FETCH_SIZE"] == 10.0


def test_json_summary_splits_by_xcc(tmp_path):
    inst = [{"dimensions": [{"dimension_name": "DIMENSION_INSTANCE", "index": i % 2},
                            {"dimension_name": "DIMENSION_XCC", "index": i // 2}]} for i in range(4)]
    doc = {"rocprofiler-sdk-tool": [{
        "counters": [{"id": {"handle": 7}, "name": "TCC_HIT", "instances": inst},
                     {"id": {"handle": 9}, "name": "TCC_MISS", "instances": inst}],
        "kernel_symbols": [{"kernel_id": 3, "formatted_kernel_name": "gemm<2>"}],
        "callback_records": {"counter_collection": [{
            "dispatch_data": {"dispatch_info": {"kernel_id": 3, "dispatch_id": 1}},
            "records": [{"counter_id": {"handle": 7}, "value": v} for v in (1, 2, 30, 40)]
                       + [{"counter_id": {"handle": 9}, "value": v} for v in (1, 0, 10, 20)]}]}}]}
    d = tmp_path / "j"
    os.makedirs(d)
    (d / "5_results.json").write_text(json.dumps(doc))
    r = harness.summarize_json(str(d), "gemm")["gemm<2>"]
    assert r["n"] == 1
    assert r["counters"]["TCC_HIT"]["total"] == 73 and r["counters"]["TCC_HIT"]["per_xcc"] == [3, 70]
    assert r["counters"]["TCC_MISS"]["per_xcc"] == [1, 30]


# ---------------------------------------------------------------------------- candidate ranking (no GPU: canned child outputs)

def _row(mode, g, tile, hit, model=80.0, panels=100, valid=True, us=100.0):
    return dict(mode=mode, group_m=g, tile=tile, valid=valid, l2_hit_pct=hit, model_hit_pct=model, model_panels=panels, us_per_launch=us)


def test_check_line_parser():
    ok = "ran 30 warm-up + 20 timed launches\ncheck: bit_identical_to_rr=True map_is_permutation=True us_per_launch=93.125\n"
    assert harness.parse_check_line(ok) == (True, 93.125)
    assert harness.parse_check_line(ok.replace("rr=True", "rr=False"))[0] is False
    assert harness.parse_check_line(ok.replace("permutation=True", "permutation=False"))[0] is False
    valid, us = harness.parse_check_line("Traceback (most recent call last):\n  boom\n")     # the child died: not a valid candidate
    assert valid is False and us != us


def test_ranking_drops_broken_remaps_and_orders_by_measured_hit_rate():
    rows = [_row("rr", None, 256, 48.5), _row("xcd", None, 256, 80.3), _row("xcd_groupm", 4, 256, 80.2),
            _row("groupm", 8, 256, 99.0, valid=False),                      # highest hit rate, but its bits differ: broken remap
            _row("groupm", 2, 256, None),                                    # profiler pass failed: no measurement
            _row("groupm", 4, 256, float("nan"))]
    good, best, tied = harness.rank_candidates(rows)
    assert [r["mode"] for r in good] == ["xcd", "xcd_groupm", "rr"]
    assert all(r["valid"] for r in good)
    # 80.3 and 80.2 are within half a point: a tie, which the library default wins although it measured 0.1 lower and is not faster
    assert (best["mode"], best["group_m"]) == ("xcd_groupm", 4) and [r["mode"] for r in tied] == ["xcd"]
    assert harness.rank_candidates([_row("rr", None, 256, 70.0, valid=False)]) == ([], None, [])


def test_ranking_ties_are_broken_by_the_panel_model_not_by_timing():
    rows = [_row("groupm", 2, 256, 79.48, panels=3000, us=90.0),             # fastest by a hair: must not matter
            _row("xcd_groupm", 8, 256, 79.47, panels=2000, us=99.0),         # fewest panels predicted: wins the tie
            _row("xcd_groupm", 4, 256, 79.40, panels=3000, us=95.0),
            _row("rr", None, 256, 70.7, panels=4000, us=89.0)]
    good, best, tied = harness.rank_candidates(rows)
    assert (best["mode"], best["group_m"]) == ("xcd_groupm", 8)
    assert {(r["mode"], r["group_m"]) for r in tied} == {("groupm", 2), ("xcd_groupm", 4)}
    # with equal predictions the library default is kept, and after it the simpler mapping
    for r in rows:
        r["model_panels"] = 3000
    _, best, _ = harness.rank_candidates(rows)
    assert (best["mode"], best["group_m"]) == ("xcd_groupm", 4)
    _, best, _ = harness.rank_candidates([r for r in rows if r["group_m"] != 4])
    assert best["mode"] == "groupm"
    # outside the tie window the measurement decides, whatever the model says
    rows[3]["l2_hit_pct"], rows[3]["model_panels"] = 85.0, 9999
    _, best, tied = harness.rank_candidates(rows)
    assert best["mode"] == "rr" and tied == []


def test_tile_shapes_are_compared_by_missed_bytes_not_by_hit_rate():
    # a 128-wide tile asks for twice the lines per flop: its hit rate reads higher although more bytes cross the fabric
    small = dict(_row("groupm", 2, 128, 82.8), l2_miss_mib=362.8)
    big = dict(_row("xcd_groupm", 4, 256, 79.5), l2_miss_mib=224.0)
    assert harness.pick_across_tiles([small, big]) is big
    assert harness.pick_across_tiles([small, None]) is small and harness.pick_across_tiles([None]) is None
    del small["l2_miss_mib"]                                                 # no measurement: the model's panel bytes decide
    small["model_panels"], big["model_panels"] = 200, 100
    assert harness.pick_across_tiles([small, big]) is big


def test_candidate_list_spans_mode_group_and_tile():
    c = harness.candidate_list([1, 4], [256, 128])
    assert len(c) == 2 * (2 + 2 * 2) and ("xcd_groupm", 4, 128) in c and ("rr", 0, 256) in c
    assert {t for _, _, t in c} == {256, 128}


def test_harness_panel_model_agrees_with_the_oracles_on_library_maps():
    # two independent implementations (the package never imports the oracle): same counts on the workload grids
    import paper_2508_20258_amd as swz
    from oracle import l2_model, pid_map as opm
    for gm, gn in [(16, 16), (32, 32), (64, 8), (40, 28), (79, 55), (4, 4), (5, 7)]:
        for mode in range(4):
            for slots in (32, 64, 5):
                lib_map = swz.pid_map(gm, gn, 8, 4, mode)
                got, distinct, requested = harness.panel_model(lib_map, gn, 8, slots)
                assert abs(got - l2_model.predicted_hit_rate(opm.pid_map(gm, gn, 8, 4, mode), gn, 8, slots)) < 1e-12
                assert requested == 2 * gm * gn and 0 < distinct <= requested
    assert harness.co_resident_tiles_per_xcd(256, 256, 8) == 32 and harness.co_resident_tiles_per_xcd(128, 256, 8) == 64


def test_recorded_counters_are_tied_to_the_kernel_sources(tmp_path, monkeypatch):
    rec = tmp_path / "measured_counters.json"
    monkeypatch.setattr(harness, "RECORD_PATH", str(rec))
    assert harness.recorded_counters() is None                                 # nothing recorded
    rec.write_text(json.dumps({"kernel_sha256": harness.kernel_hash(), "workloads": {"cfg2_4096": {"rr": {"l2_hit_pct": 70.7}}}}))
    assert harness.recorded_counters("cfg2_4096")["rr"]["l2_hit_pct"] == 70.7
    assert harness.recorded_counters("cfg3_8192") is None
    rec.write_text(json.dumps({"kernel_sha256": "0" * 64, "workloads": {"cfg2_4096": {}}}))
    assert harness.recorded_counters("cfg2_4096") is None                      # another kernel's counters are not reported


def test_csv_summary_last_n(tmp_path):
    d = tmp_path / "run"
    os.makedirs(d)
    rows = "".join(f'"KERNEL_DISPATCH","gemm<2>",{1000 * i},{1000 * i + (500 if i < 6 else 100)}\n' for i in range(10))
    (d / "1_kernel_trace.csv").write_text('"Kind","Kernel_Name","Start_Timestamp","End_Timestamp"\n' + rows)
    assert harness.summarize(str(d), "gemm", last=4)["gemm<2>"]["warm_avg_ns"] == 100       # the timed launches only
    assert harness.summarize(str(d), "gemm")["gemm<2>"]["warm_avg_ns"] == (500 + 4 * 100) / 5
    assert len(harness.summarize_spans(str(d), "gemm")) == 10


def test_clocks_report_on_hand_made_stamps():
    import numpy as np
    # two XCDs, two workgroups each; XCD 1 runs its loop at 1500 MHz, XCD 0 at 2000 MHz; 100 steps of 1100 cycles
    rows = []
    for w in range(4):
        x = w % 2
        mhz = 2000 if x == 0 else 1500
        cyc = 100 * 1100
        ticks = int(round(cyc / mhz * 100))                  # 100 MHz ticks the loop lasts
        c0, r0 = 10_000 + w, 500 + w
        rows.append([c0, r0, c0 + 4000, r0 + 200, c0 + 4000 + cyc, r0 + 200 + ticks, c0 + 4000 + cyc + 2000, r0 + 200 + ticks + 100,
                     x, 0, 100, w // 2, w % 2, 0, 0, 0])
    text = harness.clocks_report(np.array(rows), 1e9, "label")
    lines = text.splitlines()
    x0 = next(l for l in lines if l.startswith("  0 ")).split()
    x1 = next(l for l in lines if l.startswith("  1 ")).split()
    assert x0[1] == "2" and float(x0[2]) == 1100.0 and abs(float(x0[5]) - 2000) <= 2
    assert float(x1[2]) == 1100.0 and abs(float(x1[5]) - 1500) <= 2
    assert float(x1[9]) > float(x0[9])                     # the slower XCD's loop lasts longer
    assert "slowest XCD 15" in lines[-1] and "fastest 20" in lines[-1]


def test_profile_table_from_canned_rocprof_output(tmp_path):
    # the table kept under profiles/ and the record bench.py reports, rebuilt from hand-made pass directories:
    # scaling of the byte counters by the copy calibration, hit rates total and per XCD, MfmaUtil, last-N kernel time
    def counters_csv(d, kernel, rows):
        os.makedirs(d)
        (d / "1_counter_collection.csv").write_text('"Dispatch_Id","Kernel_Name","Counter_Name","Counter_Value"\n' +
                                                    "".join(f'{i},"{kernel}","{c}",{v}\n' for i, c, v in rows))

    src = tmp_path / "prof"
    counters_csv(src / "copy_fetch", "copy16_kernel", [(1, "FETCH_SIZE", 524288.0)])      # reads half the KiB copied -> x2
    counters_csv(src / "copy_write", "copy16_kernel", [(1, "WRITE_SIZE", 1048576.0)])     # -> x1
    inst = [{"dimensions": [{"dimension_name": "DIMENSION_XCC", "index": x}]} for x in range(8)]
    for mode, (hit, miss) in {"rr": (70, 30), "xcd": (70, 30), "xcd_groupm": (80, 20)}.items():
        t = src / f"cfg1_512_{mode}"
        kt = tmp_path / "prof" / f"cfg1_512_{mode}_kt"
        os.makedirs(kt)
        rows = "".join(f'"KERNEL_DISPATCH","gemm_bf16_kernel<{mode}>",{1000 * i},{1000 * i + (900 if i < 30 else 500)}\n' for i in range(40))
        (kt / "1_kernel_trace.csv").write_text('"Kind","Kernel_Name","Start_Timestamp","End_Timestamp"\n' + rows)
        (tmp_path / "prof" / f"cfg1_512_{mode}_kt.log").write_text("ran 30 warm-up + 10 timed launches of cfg1_512 mode x: 0.61 us per launch\n")
        tcc = tmp_path / "prof" / f"cfg1_512_{mode}_tcc"
        os.makedirs(tcc)
        doc = {"rocprofiler-sdk-tool": [{
            "counters": [{"id": {"handle": 1}, "name": "TCC_HIT", "instances": inst}, {"id": {"handle": 2}, "name": "TCC_MISS", "instances": inst}],
            "kernel_symbols": [{"kernel_id": 5, "formatted_kernel_name": "gemm_bf16_kernel"}],
            "callback_records": {"counter_collection": [{"dispatch_data": {"dispatch_info": {"kernel_id": 5}},
                                                        "records": [{"counter_id": {"handle": 1}, "value": hit + x} for x in range(8)]
                                                        + [{"counter_id": {"handle": 2}, "value": miss - x} for x in range(8)]}]}}]}
        (tcc / "1_results.json").write_text(json.dumps(doc))
        counters_csv(tmp_path / "prof" / f"cfg1_512_{mode}_fetch", "gemm_bf16_kernel", [(1, "FETCH_SIZE", 1536.0)])
        counters_csv(tmp_path / "prof" / f"cfg1_512_{mode}_write", "gemm_bf16_kernel", [(1, "WRITE_SIZE", 512.0)])
        counters_csv(tmp_path / "prof" / f"cfg1_512_{mode}_sq", "gemm_bf16_kernel",
                     [(1, "SQ_VALU_MFMA_BUSY_CYCLES", 512000.0), (1, "GRBM_GUI_ACTIVE", 8000.0), (1, "SQ_INSTS_VALU_MFMA_MOPS_BF16", 524288.0),
                      (1, "SQ_LDS_BANK_CONFLICT", 0.0), (1, "SQ_LDS_IDX_ACTIVE", 100.0), (1, "SQ_BUSY_CU_CYCLES", 1.0), (1, "SQ_WAVE_CYCLES", 1.0)])
    text, record = harness.profile_table(str(src), "cfg1_512", 40.0, 10)
    r = record["xcd_groupm"]
    assert r["kernel_us"] == 0.5                                             # the last 10 dispatches, not the 30 slower ones before
    assert abs(r["l2_hit_pct"] - 100 * (8 * 80 + 28) / 800) < 1e-9           # sum over the instances
    assert abs(r["l2_hit_pct_per_xcd"][3] - 83.0) < 1e-9 and len(r["l2_hit_pct_per_xcd"]) == 8
    assert r["fetch_bytes"] == 1536 * 2 * 1024 and r["write_bytes"] == 512 * 1024   # scaled by the copy calibration
    assert abs(r["mfma_util_pct"] - 100 * 512000 / (8000 / 8 * 1024)) < 1e-9
    assert r["mfma_flop_issued"] == 524288 * 512 == 2 * 512 ** 3
    assert abs(record["rr"]["model_hit_pct"] - 25.0) < 1e-9                  # 4 x 4 grid, two tiles per XCD: nothing shared beyond 2 of 8 requests
    line = next(l for l in text.splitlines() if l.startswith("xcd_groupm"))
    assert line.split()[1] == "0.50" and line.split()[2] == "0.90" and line.split()[4] == "0.61"
    assert "scale FETCH_SIZE by 2.000, WRITE_SIZE by 1.000" in text
