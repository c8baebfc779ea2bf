"""Pins for the constructive PID-map oracle: each checks it against something other than itself."""
import itertools
import os

import pytest

from oracle import pid_map as opm

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def paper_printed_swizzle(pid, num_blocks, num_xcds):
    # The closed form printed in the paper's GEMM appendix figure (ceil-divided blocks per XCD).
    b_per_xcd = (num_blocks + num_xcds - 1) // num_xcds
    return (pid % num_xcds) * b_per_xcd + pid // num_xcds


def test_worked_example_4x5_on_4_xcds():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "gemm_swizzle_4x5_xcd4.txt")) if not l.startswith("#")]
    want = [int(t) for _, t in rows]
    assert [int(w) for w, _ in rows] == list(range(20))
    assert opm.pid_map(4, 5, 4, 1, opm.MODE_XCD) == want
    # the point of the example: every XCD owns one whole tile-row of C (shares A's row panel)
    for x, tiles in enumerate(opm.xcd_tile_sets(want, 4)):
        assert {t // 5 for t in tiles} == {x}


@pytest.mark.parametrize("num_blocks,num_xcds", [(304, 8), (256, 8), (1024, 8), (512, 8), (1120, 8), (20, 4),
                                                 (16, 8), (96, 12), (7, 7), (35, 5)])
def test_equals_paper_formula_when_divisible(num_blocks, num_xcds):
    assert num_blocks % num_xcds == 0
    want = [paper_printed_swizzle(w, num_blocks, num_xcds) for w in range(num_blocks)]
    assert opm.logical_ids(num_blocks, num_xcds, True) == want


def test_paper_formula_is_not_a_bijection_on_ragged_counts_and_checker_says_so():
    bad = [paper_printed_swizzle(w, 10, 8) for w in range(10)]
    assert bad == [0, 2, 4, 6, 8, 10, 12, 14, 1, 3]
    assert not opm.is_permutation(bad, 10)
    # ... whereas the dealt-and-numbered map is
    assert opm.is_permutation(opm.logical_ids(10, 8, True), 10)


def test_checker_rejects_bit_swap_remap_on_non_power_of_two():
    # the "hardware-overload" pattern printed in the paper's bitwise-swizzling appendix
    def swap(pid):
        return ((pid >> 1) & 0x55555555) | ((pid & 0x55555555) << 1)
    assert opm.is_permutation([swap(p) for p in range(16)], 16)       # fine on 16
    assert not opm.is_permutation([swap(p) for p in range(21)], 21)   # sends 20 -> 24
    assert not opm.is_permutation([0, 1, 1, 3], 4)
    assert not opm.is_permutation([0, 1, 2], 4)
    assert not opm.is_permutation([0, 1, 2, -1], 4)


@pytest.mark.parametrize("T,X", [(t, x) for t in range(1, 70) for x in range(1, 13)])
def test_xcd_numbering_is_the_rank_under_sorting_by_xcd_then_launch_order(T, X):
    # Independent route: sort the workgroups by (XCD they land on, launch order); rank = logical id.
    by_xcd = sorted(range(T), key=lambda w: (w % X, w))
    want = [0] * T
    for rank, w in enumerate(by_xcd):
        want[w] = rank
    assert opm.logical_ids(T, X, True) == want


@pytest.mark.parametrize("gm,gn,g", [(gm, gn, g) for gm in range(1, 11) for gn in range(1, 8) for g in (1, 2, 3, 4, 5, 11)])
def test_grouped_raster_is_the_sort_by_band_column_row(gm, gn, g):
    want = sorted(((pm, pn) for pm in range(gm) for pn in range(gn)), key=lambda t: (t[0] // g, t[1], t[0]))
    assert opm.raster_order(gm, gn, g, True) == want
    assert opm.raster_order(gm, gn, g, False) == sorted((pm, pn) for pm in range(gm) for pn in range(gn))


def test_special_cases():
    for gm, gn in [(3, 7), (8, 8), (5, 5), (1, 9), (9, 1)]:
        T = gm * gn
        rowmajor = list(range(T))
        colmajor = [pm * gn + pn for pn in range(gn) for pm in range(gm)]
        assert opm.pid_map(gm, gn, 8, 4, opm.MODE_RR) == rowmajor
        assert opm.pid_map(gm, gn, 1, 4, opm.MODE_XCD) == rowmajor            # one XCD: nothing to renumber
        assert opm.pid_map(gm, gn, 8, 1, opm.MODE_GROUPM) == rowmajor         # bands of one row
        assert opm.pid_map(gm, gn, 1, gm, opm.MODE_XCD_GROUPM) == colmajor    # one band: column-major
        assert opm.pid_map(gm, gn, 8, gm + 3, opm.MODE_GROUPM) == colmajor
        assert opm.pid_map(gm, gn, T + 5, 4, opm.MODE_XCD) == rowmajor        # fewer workgroups than XCDs
        assert opm.pid_map(gm, gn, 8, 1, opm.MODE_XCD_GROUPM) == opm.pid_map(gm, gn, 8, 1, opm.MODE_XCD)


@pytest.mark.parametrize("gm,gn", [(4, 4), (16, 16), (32, 32), (64, 8), (40, 28), (79, 55), (79, 28), (5, 5), (7, 3), (1, 1), (2, 3)])
@pytest.mark.parametrize("X", [1, 3, 4, 8])
@pytest.mark.parametrize("mode", [0, 1, 2, 3])
def test_invariants(gm, gn, X, mode):
    g = 4
    out = opm.pid_map(gm, gn, X, g, mode)
    T = gm * gn
    assert opm.is_permutation(out, T)
    assert opm.fair_share(out, gm, gn, g, mode in (2, 3), X, mode in (1, 2))
    if mode in (1, 2):
        assert opm.xcd_runs_contiguous(out, gm, gn, g, mode == 2, X)
    if mode == 2:
        # along the logical order, every aligned run inside a band stays in one tile column
        inv = sorted(range(T), key=lambda w: opm.logical_ids(T, X, True)[w])
        seq = [out[w] for w in inv]
        assert seq == [pm * gn + pn for pm, pn in opm.raster_order(gm, gn, g, True)]


def test_checkers_catch_planted_mistakes():
    gm, gn, X, g = 6, 5, 4, 2
    good = opm.pid_map(gm, gn, X, g, 2)
    assert opm.xcd_runs_contiguous(good, gm, gn, g, True, X)
    swapped = list(good)
    swapped[0], swapped[1] = swapped[1], swapped[0]          # still a permutation, but XCD 0 and 1 trade a tile
    assert opm.is_permutation(swapped, gm * gn)
    assert not opm.xcd_runs_contiguous(swapped, gm, gn, g, True, X)
    rr = opm.pid_map(gm, gn, X, g, 0)
    assert not opm.xcd_runs_contiguous(rr, gm, gn, g, False, X)   # round-robin scatters neighbours


def test_fair_share_checker_can_fail():
    # Each planted map breaks the invariant in a different way; the checker must reject every one of them
    # and accept the maps they were derived from.
    gm, gn, X, g = 6, 5, 4, 2                      # T = 30 = 4*7 + 2: XCDs 0, 1 hold 8 raster positions, XCDs 2, 3 hold 7
    T = gm * gn
    for mode in range(4):
        good = opm.pid_map(gm, gn, X, g, mode)
        args = (gm, gn, g, mode in (2, 3), X)
        assert opm.fair_share(good, *args, mode in (1, 2))
        # XCD 0 is handed one of XCD 1's tiles (that tile is then computed twice, one of XCD 0's never)
        stolen = list(good)
        stolen[0] = good[1]
        assert not opm.fair_share(stolen, *args, False)
        # right length, not a permutation: a tile repeated inside one XCD's own share
        repeated = list(good)
        repeated[X] = good[0]
        assert not opm.fair_share(repeated, *args, False)
        # wrong lengths: an XCD loses its workgroups / a stray extra workgroup
        lopsided = [t for w, t in enumerate(good) if w % X != 1]
        assert not opm.fair_share(lopsided, *args, False)
        assert not opm.fair_share(good + [good[0]], *args, False)
        assert not opm.fair_share(good[:-1], *args, False)
        # a tile outside the grid
        outside = list(good)
        outside[3] = T
        assert not opm.fair_share(outside, *args, False)
    # a permutation in which two XCDs trade a tile: counts are right, so the plain share check passes,
    # but XCD 0's share no longer is the stretch of the raster that begins at 0 / XCD 1's at 8
    good = opm.pid_map(gm, gn, X, g, 2)
    traded = list(good)
    traded[0], traded[1] = traded[1], traded[0]
    assert opm.is_permutation(traded, T) and opm.fair_share(traded, gm, gn, g, True, X, False)
    assert not opm.fair_share(traded, gm, gn, g, True, X, True)
    # round-robin dispatch of the plain raster is fair in counts but no XCD's share begins where the previous ends
    rr = opm.pid_map(gm, gn, X, g, 0)
    assert opm.fair_share(rr, gm, gn, g, False, X, False) and not opm.fair_share(rr, gm, gn, g, False, X, True)
    # the paper's printed ceil-form on a ragged count leaves [0, T) and must fail too
    bad = [paper_printed_swizzle(w, 10, 8) for w in range(10)]
    assert not opm.fair_share(bad, 2, 5, 1, False, 8, True)
    # random lists of the right length (what the old length-only check accepted) fail
    import random
    rng = random.Random(5)
    assert not any(opm.fair_share([rng.randrange(T) for _ in range(T)], gm, gn, g, False, X, False) for _ in range(50))


@pytest.mark.parametrize("T,X", [(20, 4), (30, 4), (10, 8), (5, 8), (4345, 8), (25, 8), (7, 7)])
def test_fair_share_sizes_against_brute_force_counts(T, X):
    # the share sizes the checker demands, counted the slow way: deal T workgroups one at a time
    counts = [0] * X
    for w in range(T):
        counts[w % X] += 1
    out = opm.pid_map(1, T, X, 1, opm.MODE_XCD)
    assert opm.fair_share(out, 1, T, 1, False, X, True)
    for x, tiles in enumerate(opm.xcd_tile_sets(out, X)):
        assert len(tiles) == counts[x] and tiles == list(range(sum(counts[:x]), sum(counts[:x + 1])))


def test_bad_arguments_raise():
    for args in [(0, 4, 8, 4, 0), (4, 0, 8, 4, 0), (4, 4, 0, 4, 1), (4, 4, 8, 0, 2), (4, 4, 8, 4, 8), (4, 4, 8, 4, -1)]:
        with pytest.raises(ValueError):
            opm.pid_map(*args)


# ---------------------------------------------------------------------------- persistent launch style

def test_persistent_map_is_the_papers_listing_on_its_own_shape():
    # the paper's kernel: num_blocks = number of compute units (304 on the part it names), 8 XCDs, and a
    # tile loop with that stride; pid = (pid % 8) * 38 + pid // 8 for 304 = 8 * 38 workgroups
    G, X = 304, 8
    gm, gn = 32, 32
    rounds = opm.pid_map_persistent(gm, gn, X, 1, opm.MODE_XCD, G)
    for i, row in enumerate(rounds):
        for w, t in enumerate(row):
            pos = paper_printed_swizzle(w, G, X) + i * G
            assert t == (pos if pos < gm * gn else -1)


@pytest.mark.parametrize("gm,gn,X,g,G", [(16, 16, 8, 4, 256), (32, 32, 8, 4, 256), (40, 28, 8, 4, 256), (5, 7, 8, 4, 6),
                                         (7, 3, 4, 2, 10), (4, 5, 4, 4, 8), (3, 3, 8, 4, 9), (9, 11, 8, 4, 30), (6, 6, 5, 3, 7)])
def test_persistent_map_invariants(gm, gn, X, g, G):
    T = gm * gn
    for mode in range(4):
        rounds = opm.pid_map_persistent(gm, gn, X, g, mode, G)
        assert len(rounds) == -(-T // G) and all(len(r) == G for r in rounds)
        tiles = [t for r in rounds for t in r if t >= 0]
        assert opm.is_permutation(tiles, T)                       # every tile exactly once
        order = opm.raster_order(gm, gn, g, mode in (2, 3))
        pos = {pm * gn + pn: l for l, (pm, pn) in enumerate(order)}
        for i, row in enumerate(rounds):
            # a workgroup never skips a round and then works again
            for w in range(G):
                if row[w] < 0:
                    assert all(r[w] < 0 for r in rounds[i:])
            if mode in (1, 2):
                # in a full round the tiles of one XCD are one contiguous run of the raster
                if all(t >= 0 for t in row):
                    for x in range(min(X, G)):
                        ps = sorted(pos[row[w]] for w in range(x, G, X))
                        assert ps == list(range(ps[0], ps[0] + len(ps)))
        if G >= T:
            # one round, and then it is the one-workgroup-per-tile map restricted to T workgroups only
            # when nothing is renumbered
            assert len(rounds) == 1
            if mode in (0, 3):
                assert rounds[0][:T] == opm.pid_map(gm, gn, X, g, mode)


def test_persistent_with_one_workgroup_per_tile_equals_the_plain_map():
    for gm, gn, X, g in [(4, 5, 4, 2), (6, 7, 8, 4), (3, 3, 8, 4)]:
        for mode in range(4):
            assert opm.pid_map_persistent(gm, gn, X, g, mode, gm * gn) == [opm.pid_map(gm, gn, X, g, mode)]


# ---------------------------------------------------------------------------- skewed raster (modes 4..7)

@pytest.mark.parametrize("gm,gn", [(1, 1), (1, 7), (7, 1), (4, 4), (5, 3), (3, 5), (8, 8), (6, 10), (16, 16), (9, 31)])
def test_skew_is_a_cyclic_roll_of_every_grid_column(gm, gn):
    # independent route: lay the unskewed raster positions out as a grid_m x grid_n array; the skew rolls
    # column c down by c (numpy's roll), nothing else
    import numpy as np
    for grouped in (False, True):
        g = 3
        plain = opm.raster_order(gm, gn, g, grouped, False)
        pos = np.full((gm, gn), -1)
        for l, (pm, pn) in enumerate(plain):
            pos[pm, pn] = l
        rolled = np.stack([np.roll(pos[:, c], c) for c in range(gn)], axis=1)
        skewed = opm.raster_order(gm, gn, g, grouped, True)
        for l, (pm, pn) in enumerate(skewed):
            assert rolled[pm, pn] == l
        assert sorted(skewed) == sorted(plain)                      # still every tile exactly once
        assert [pn for _, pn in skewed] == [pn for _, pn in plain]  # tiles never change their column


def test_skew_special_cases_and_the_diagonal_property():
    # one column: nothing moves; skew of a square row-major raster: every raster row is a full diagonal
    assert opm.raster_order(6, 1, 2, False, True) == opm.raster_order(6, 1, 2, False, False)
    n = 8
    order = opm.raster_order(n, n, 1, False, True)
    for r in range(n):
        row = order[r * n:(r + 1) * n]
        assert sorted(pm for pm, _ in row) == list(range(n)) and [pn for _, pn in row] == list(range(n))
        assert row[0] == (r, 0) and row[1] == ((r + 1) % n, 1)
    # inside one raster row, a window of consecutive positions touches as many tile rows as tile columns (up to grid_m)
    for gm, gn, width in [(16, 16, 10), (128, 128, 40), (5, 9, 9), (9, 5, 5), (3, 8, 6)]:
        order = opm.raster_order(gm, gn, 1, False, True)
        for r in range(gm):
            for c0 in range(gn - width + 1):
                w = order[r * gn + c0:r * gn + c0 + width]
                assert len({pn for _, pn in w}) == width and len({pm for pm, _ in w}) == min(width, gm)
    # the worked 4 x 5 example with the skew on top: XCD x, which owned tile row x, now owns a diagonal
    want = [((x + c) % 4) * 5 + c for x in range(4) for c in range(5)]
    got = opm.pid_map(4, 5, 4, 1, opm.MODE_XCD + opm.MODE_SKEW)
    assert [got[w] for x in range(4) for w in range(x, 20, 4)] == want


@pytest.mark.parametrize("gm,gn", [(4, 4), (16, 16), (40, 28), (79, 55), (5, 5), (7, 3), (1, 1), (2, 3), (128, 128)])
@pytest.mark.parametrize("X", [1, 3, 8])
@pytest.mark.parametrize("mode", [4, 5, 6, 7])
def test_invariants_of_skewed_modes(gm, gn, X, mode):
    g = 4
    out = opm.pid_map(gm, gn, X, g, mode)
    renumber, grouped, skewed = opm.mode_parts(mode)
    assert skewed and opm.is_permutation(out, gm * gn)
    assert opm.fair_share(out, gm, gn, g, grouped, X, renumber, skewed=True)
    if renumber:
        assert opm.xcd_runs_contiguous(out, gm, gn, g, grouped, X, skewed=True)
        if gn > 1 and gm > 1:
            assert not opm.xcd_runs_contiguous(out, gm, gn, g, grouped, X, skewed=False) or gm * gn <= X
    # the skewed map is the unskewed one with every tile moved down its column, cyclically
    plain = opm.pid_map(gm, gn, X, g, mode - 4)
    assert out == [((t // gn + t % gn) % gm) * gn + t % gn for t in plain]


def test_mode_parts_and_bad_modes():
    assert [opm.mode_parts(m) for m in range(8)] == [(False, False, False), (True, False, False), (True, True, False),
                                                     (False, True, False), (False, False, True), (True, False, True),
                                                     (True, True, True), (False, True, True)]
    for bad in (-1, 8, 12):
        with pytest.raises(ValueError):
            opm.pid_map(4, 4, 8, 4, bad)
        with pytest.raises(ValueError):
            opm.pid_map_persistent(4, 4, 8, 4, bad, 8)
    rounds = opm.pid_map_persistent(5, 7, 8, 2, 6, 6)
    assert opm.is_permutation([t for r in rounds for t in r if t >= 0], 35)
