"""Property tests: the library's closed-form PID maps against the constructive oracle on random grids."""
import numpy as np
from hypothesis import given, settings, strategies as st

import paper_2508_20258_amd as swz
from oracle import pid_map as opm

grid = st.integers(min_value=1, max_value=70)
xcd = st.integers(min_value=1, max_value=17)
grp = st.integers(min_value=1, max_value=80)
mode = st.integers(min_value=0, max_value=7)


@settings(max_examples=300, deadline=None)
@given(grid, grid, xcd, grp, mode)
def test_one_workgroup_per_tile(gm, gn, X, g, m):
    got = swz.pid_map(gm, gn, X, g, m)
    assert got.tolist() == opm.pid_map(gm, gn, X, g, m)
    assert np.array_equal(np.sort(got), np.arange(gm * gn))          # bijection onto [0, T)
    renumber, grouped, skewed = opm.mode_parts(m)
    assert opm.fair_share(got.tolist(), gm, gn, g, grouped, X, renumber, skewed)
    if renumber:
        assert opm.xcd_runs_contiguous(got.tolist(), gm, gn, g, grouped, X, skewed)


@settings(max_examples=200, deadline=None)
@given(grid, grid, xcd, grp, mode, st.integers(min_value=1, max_value=300))
def test_persistent(gm, gn, X, g, m, G):
    got = swz.pid_map_persistent(gm, gn, X, g, m, G)
    assert got.tolist() == opm.pid_map_persistent(gm, gn, X, g, m, G)
    tiles = got[got >= 0]
    assert np.array_equal(np.sort(tiles), np.arange(gm * gn))        # every tile exactly once
    assert set(np.unique(got[got < 0]).tolist()) <= {-1}


def test_large_grids_stay_bijective():
    # beyond what the oracle's lists are comfortable with: check the invariant only
    for gm, gn, X, g in [(1000, 999, 8, 4), (4096, 257, 8, 16), (3, 200000, 7, 2), (46340, 46340 // 100, 8, 4)]:
        for m in range(8):
            got = swz.pid_map(gm, gn, X, g, m)
            seen = np.zeros(gm * gn, dtype=bool)
            seen[got] = True
            assert seen.all() and got.min() == 0 and got.max() == gm * gn - 1
