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
