"""Host-side checks of libswz that need no GPU: exports, the closed-form PID map, error paths."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2508_20258_amd as swz
from oracle import pid_map as opm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_entry_point():
    header = open(os.path.join(ROOT, "include", "swz.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(swz_[a-z_]+)\s*\(", header))
    assert declared == {"swz_status_string", "swz_device_info", "swz_pid_map", "swz_pid_map_device", "swz_gemm",
                        "swz_gemm_ex", "swz_gemm_plan", "swz_copy_bytes", "swz_pid_map_persistent",
                        "swz_pid_map_persistent_device", "swz_transpose", "swz_softmax", "swz_layernorm", "swz_mfma_peak",
                        "swz_gemm_probe"}
    raw = ctypes.CDLL(swz.binding.LIB_PATH)
    for name in declared:
        assert hasattr(raw, name), name
    assert set(swz.binding.EXPORTS) == declared


GRIDS = [(gm, gn) for gm in range(1, 13) for gn in range(1, 13)]


@pytest.mark.parametrize("mode", [0, 1, 2, 3, 4, 5, 6, 7])
def test_closed_form_equals_constructive_oracle_exhaustively(mode):
    for gm, gn in GRIDS:
        for X in range(1, 13):
            for g in range(1, 14):
                got = swz.pid_map(gm, gn, X, g, mode).tolist()
                assert got == opm.pid_map(gm, gn, X, g, mode), (gm, gn, X, g, mode)


@pytest.mark.parametrize("gm,gn,X,g", [(4, 4, 8, 4), (16, 16, 8, 4), (32, 32, 8, 4), (64, 8, 8, 4), (40, 28, 8, 4),
                                       (79, 55, 8, 4), (79, 28, 8, 4), (5, 5, 8, 4), (7, 3, 8, 4), (4, 5, 4, 4),
                                       (128, 96, 8, 16), (65, 67, 7, 5), (1, 300, 8, 4), (300, 1, 8, 4)])
def test_workload_grids_match_oracle_and_invariants(gm, gn, X, g):
    for mode in range(8):
        got = swz.pid_map(gm, gn, X, g, mode).tolist()
        assert got == opm.pid_map(gm, gn, X, g, mode)
        renumber, grouped, skewed = opm.mode_parts(mode)
        assert opm.is_permutation(got, gm * gn) and opm.fair_share(got, gm, gn, g, grouped, X, renumber, skewed)
        if renumber:
            assert opm.xcd_runs_contiguous(got, gm, gn, g, grouped, X, skewed)


def test_error_paths_leave_output_untouched():
    L = swz.lib
    out = np.full(16, -7, dtype=np.int32)
    for args in [(0, 4, 8, 4, 0), (4, 0, 8, 4, 0), (4, 4, 0, 4, 1), (4, 4, 8, 0, 2), (4, 4, 8, 4, 8), (4, 4, 8, 4, -1),
                 (-3, 4, 8, 4, 0)]:
        assert L.swz_pid_map(*args, out.ctypes.data) == -1
        assert (out == -7).all()
    assert L.swz_pid_map(4, 4, 8, 4, 0, None) == -1
    assert L.swz_pid_map(1 << 16, 1 << 15, 8, 4, 0, out.ctypes.data) == -3       # 2^31 tiles
    assert (out == -7).all()
    with pytest.raises(swz.SwzError) as e:
        swz.pid_map(4, 4, 8, 4, 9)
    assert e.value.status == -1
    assert swz.status_string(0) == "ok" and "unknown" in swz.status_string(-99)
    for s in (-1, -2, -3, -4):
        assert swz.status_string(s) and "unknown" not in swz.status_string(s)


def test_group_m_larger_than_grid_is_one_band():
    assert swz.pid_map(5, 7, 8, 1 << 30, 3).tolist() == opm.pid_map(5, 7, 8, 5, 3)


def test_plan_resolves_tiles_without_a_device_when_num_xcd_is_given():
    p = swz.gemm_plan(512, 512, 512, num_xcd=8)
    assert (p["bm"], p["bn"], p["bk"], p["grid_m"], p["grid_n"], p["group_m"]) == (128, 128, 64, 4, 4, 4)
    p = swz.gemm_plan(10000, 7000, 4096, num_xcd=8)
    assert (p["bm"], p["grid_m"], p["grid_n"]) == (256, 40, 28)
    # grids far from the device's CU count are decided without asking a device: tiny -> 128-wide, huge -> 256-wide
    assert swz.gemm_plan(1024, 1024, 64, num_xcd=8)["bm"] == 128 and swz.gemm_plan(8192, 8192, 64, num_xcd=8)["bm"] == 256
    p = swz.gemm_plan(10000, 7000, 4096, num_xcd=8, bm=128, bn=256)
    assert (p["bm"], p["bn"], p["grid_m"], p["grid_n"]) == (128, 256, 79, 28)
    p = swz.gemm_plan(10000, 7000, 4096, num_xcd=8, bm=256, bn=128)
    assert (p["grid_m"], p["grid_n"]) == (40, 55)
    p = swz.gemm_plan(10000, 7000, 4096, num_xcd=8, bm=128, bn=128)
    assert (p["grid_m"], p["grid_n"]) == (79, 55)
    for bad in [dict(bm=64, bn=64), dict(bm=256, bn=64), dict(bm=512, bn=256), dict(bk=32)]:
        with pytest.raises(swz.SwzError) as e:
            swz.gemm_plan(1024, 1024, 1024, num_xcd=8, **bad)
        assert e.value.status == -2
    with pytest.raises(swz.SwzError) as e:
        swz.gemm_plan(0, 8, 8, num_xcd=8)
    assert e.value.status == -1
    with pytest.raises(swz.SwzError) as e:
        swz.gemm_plan(1 << 31, 8, 8, num_xcd=8)
    assert e.value.status == -3


def test_gemm_rejects_bad_arguments_before_touching_the_device():
    L = swz.lib
    p = swz.SwzParams(0, 0, 0, 0, 8)
    ref = ctypes.byref(p)
    A, B, C = 0x1000, 0x2000, 0x3000      # never dereferenced: every call below fails validation first
    assert L.swz_gemm_ex(None, B, C, 64, 64, 64, 0, 0, ref, None) == -1
    assert L.swz_gemm_ex(A, B, None, 64, 64, 64, 0, 0, ref, None) == -1
    assert L.swz_gemm_ex(A, B, C, 0, 64, 64, 0, 0, ref, None) == -1
    assert L.swz_gemm_ex(A, B, C, 64, 64, 64, 0, 8, ref, None) == -1
    assert L.swz_gemm_ex(A, B, C, 64, 64, 64, 1, 0, ref, None) == -2          # dtype
    assert L.swz_gemm_ex(A, B, C, 64, 64, 60, 0, 0, ref, None) == -2          # K % 8
    assert L.swz_gemm_ex(A, B, C, 64, 60, 64, 0, 0, ref, None) == -2          # N % 8
    assert L.swz_gemm_ex(A + 2, B, C, 64, 64, 64, 0, 0, ref, None) == -2      # alignment
    assert L.swz_gemm_ex(A, B, C, 1 << 31, 64, 64, 0, 0, ref, None) == -3


def test_persistent_closed_form_equals_constructive_oracle():
    for gm in range(1, 9):
        for gn in range(1, 9):
            for X in (1, 3, 4, 8):
                for G in (1, 2, 5, 8, 12, 64):
                    for mode in range(8):
                        got = swz.pid_map_persistent(gm, gn, X, 3, mode, G).tolist()
                        assert got == opm.pid_map_persistent(gm, gn, X, 3, mode, G), (gm, gn, X, G, mode)
    for gm, gn in [(16, 16), (32, 32), (64, 8), (40, 28), (79, 55)]:
        for mode in range(8):
            assert swz.pid_map_persistent(gm, gn, 8, 4, mode, 256).tolist() == opm.pid_map_persistent(gm, gn, 8, 4, mode, 256)


def test_persistent_error_paths():
    L = swz.lib
    out = np.full(64, -7, dtype=np.int32)
    assert L.swz_pid_map_persistent(4, 4, 8, 4, 0, 0, out.ctypes.data) == -1
    assert L.swz_pid_map_persistent(4, 4, 8, 4, 0, -3, out.ctypes.data) == -1
    assert L.swz_pid_map_persistent(4, 4, 8, 4, 8, 8, out.ctypes.data) == -1
    assert L.swz_pid_map_persistent(4, 4, 8, 4, 0, 8, None) == -1
    assert (out == -7).all()
    p = swz.gemm_plan(8192, 8192, 8192, num_xcd=8, persistent=1, num_wg=256)
    assert (p["persistent"], p["num_wg"]) == (1, 256)
    p = swz.gemm_plan(512, 512, 512, num_xcd=8, persistent=1, num_wg=256)
    assert p["num_wg"] == 16                                   # never more workgroups than tiles
    p = swz.gemm_plan(512, 512, 512, num_xcd=8)
    assert (p["persistent"], p["num_wg"]) == (0, 0)
    with pytest.raises(swz.SwzError):
        swz.gemm_plan(512, 512, 512, num_xcd=8, persistent=2)


def test_build_script_runs_without_importing_the_package():
    # the package refuses to import without libswz.so, so the build entry must not depend on importing it
    import importlib.util
    path = os.path.join(ROOT, "paper_2508_20258_amd", "build.py")
    spec = importlib.util.spec_from_file_location("swz_build_under_test", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    assert mod.build(force=False) == swz.binding.LIB_PATH          # up to date: returns without compiling
    entry = open(os.path.join(ROOT, "__graft_entry__.py")).read()
    assert "from paper_2508_20258_amd.build import" not in entry


def test_binding_refuses_tensors_of_another_device(monkeypatch):
    # the library launches on the current device; a tensor living elsewhere must be caught before the call
    import types

    import torch
    monkeypatch.setattr(torch.cuda, "current_device", lambda: 0)
    here = types.SimpleNamespace(device=types.SimpleNamespace(index=0))
    there = types.SimpleNamespace(device=types.SimpleNamespace(index=1))
    swz.binding._same_current_device(None, here, here)
    with pytest.raises(ValueError):
        swz.binding._same_current_device(None, here, there)
    with pytest.raises(ValueError):
        swz.binding._same_current_device(there, here)
    swz.binding._same_current_device(here, here)
