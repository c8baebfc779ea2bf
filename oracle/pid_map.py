"""Constructive reference for the workgroup-ID -> output-tile map (test infrastructure only).

What is modelled (SwizzlePerf, Introduction and Appendix "Case Study: GEMM Swizzling"):
the hardware hands workgroup ``w`` of a 1-D launch to XCD ``w mod X`` (round-robin), and the
swizzle renumbers workgroups so that each XCD ends up owning one contiguous run of logical
tile ids ("all contiguous blocks on the same XCD before moving to the next XCD").

The paper's printed closed form only covers launches whose size is a multiple of X, so this
oracle does not use a formula at all: it literally deals the workgroups to the XCDs and then
numbers them XCD by XCD.  The grouped-M raster (not in the paper; a band of ``group_m`` tile
rows is walked column by column before the next band starts) is likewise built as an explicit
list.  No closed form of the library appears in this file.

Modes: 0 = identity + row-major, 1 = XCD renumbering + row-major,
       2 = XCD renumbering + grouped-M, 3 = identity + grouped-M;
       + 4 (MODE_SKEW) = the same with a skewed raster: column pn of the tile grid is shifted down
       cyclically by pn tile rows, so a run of consecutive raster positions that used to stay in one
       tile row now walks a diagonal and touches as many different tile rows as tile columns.  Not in
       the paper either: it is aimed at the memory channels, not at the L2 (a transpose of a matrix
       whose row pitch is a power of two writes a whole tile row's worth of tiles into the same few
       channels); as a PID remap it is judged by the paper's own criterion, bijectivity.
"""
from __future__ import annotations

MODE_RR, MODE_XCD, MODE_XCD_GROUPM, MODE_GROUPM = 0, 1, 2, 3
MODE_SKEW = 4
VALID_MODES = tuple(range(8))


def mode_parts(mode: int) -> tuple[bool, bool, bool]:
    """(XCD renumbering?, grouped-M raster?, skewed raster?) of a mode."""
    base = mode % 4
    return base in (MODE_XCD, MODE_XCD_GROUPM), base in (MODE_XCD_GROUPM, MODE_GROUPM), mode >= MODE_SKEW


def deal_round_robin(num_wg: int, num_xcd: int) -> list[list[int]]:
    """Hardware dispatch: bucket[x] lists, in launch order, the workgroups that XCD x receives."""
    buckets: list[list[int]] = [[] for _ in range(num_xcd)]
    for w in range(num_wg):
        buckets[w % num_xcd].append(w)
    return buckets


def logical_ids(num_wg: int, num_xcd: int, xcd_remap: bool) -> list[int]:
    """l[w]: the logical id workgroup w works on."""
    if not xcd_remap:
        return list(range(num_wg))
    l_of_w = [-1] * num_wg
    nxt = 0
    for bucket in deal_round_robin(num_wg, num_xcd):   # XCD 0 first, then XCD 1, ...
        for w in bucket:                               # inside an XCD: dispatch order
            l_of_w[w] = nxt
            nxt += 1
    return l_of_w


def shift_columns_down(order: list[tuple[int, int]], grid_m: int) -> list[tuple[int, int]]:
    """The skew: every tile of column pn moves down pn tile rows, wrapping around at the bottom."""
    moved = []
    for pm, pn in order:
        new_row = pm
        for _ in range(pn):                             # one row at a time, so that nothing but "down, wrap" is used
            new_row += 1
            if new_row == grid_m:
                new_row = 0
        moved.append((new_row, pn))
    return moved


def raster_order(grid_m: int, grid_n: int, group_m: int, grouped: bool, skewed: bool = False) -> list[tuple[int, int]]:
    """order[l] = (pm, pn): the tile visited l-th."""
    order: list[tuple[int, int]] = []
    if not grouped:
        for pm in range(grid_m):
            for pn in range(grid_n):
                order.append((pm, pn))
    else:
        first = 0
        while first < grid_m:
            rows_in_band = min(group_m, grid_m - first)     # the last band may be shorter
            for pn in range(grid_n):
                for pm in range(first, first + rows_in_band):
                    order.append((pm, pn))
            first += group_m
    return shift_columns_down(order, grid_m) if skewed else order


def pid_map(grid_m: int, grid_n: int, num_xcd: int, group_m: int, mode: int) -> list[int]:
    """out[w] = pm * grid_n + pn, the output tile that hardware workgroup w computes."""
    if grid_m < 1 or grid_n < 1 or num_xcd < 1 or group_m < 1 or mode not in VALID_MODES:
        raise ValueError("bad arguments")
    num_wg = grid_m * grid_n
    renumber, grouped, skewed = mode_parts(mode)
    l_of_w = logical_ids(num_wg, num_xcd, xcd_remap=renumber)
    order = raster_order(grid_m, grid_n, group_m, grouped, skewed)
    out = []
    for w in range(num_wg):
        pm, pn = order[l_of_w[w]]
        out.append(pm * grid_n + pn)
    return out


def pid_map_persistent(grid_m: int, grid_n: int, num_xcd: int, group_m: int, mode: int, num_wg: int) -> list[list[int]]:
    """Persistent launch (the paper's own GEMM listing: as many workgroups as compute units, each
    looping over tiles).  rounds[i][w] = tile workgroup w computes in round i, or -1.

    The workgroups (not the tiles) are dealt to the XCDs and renumbered XCD by XCD; workgroup w with
    new number p then takes the raster positions p, p + num_wg, p + 2*num_wg, ...
    """
    if grid_m < 1 or grid_n < 1 or num_xcd < 1 or group_m < 1 or num_wg < 1 or mode not in VALID_MODES:
        raise ValueError("bad arguments")
    total = grid_m * grid_n
    renumber, grouped, skewed = mode_parts(mode)
    p_of_w = logical_ids(num_wg, num_xcd, xcd_remap=renumber)
    order = raster_order(grid_m, grid_n, group_m, grouped, skewed)
    rounds = []
    start = 0
    while start < total:
        row = []
        for w in range(num_wg):
            pos = start + p_of_w[w]
            if pos < total:
                pm, pn = order[pos]
                row.append(pm * grid_n + pn)
            else:
                row.append(-1)
        rounds.append(row)
        start += num_wg
    return rounds


# ----------------------------------------------------------------------------------------
# Invariant checkers: they judge ANY candidate map (the oracle's, the library's, a broken one).
# ----------------------------------------------------------------------------------------

def is_permutation(out, num_wg: int) -> bool:
    """True iff out is a bijection onto [0, num_wg) (the paper's pass/fail criterion for a remap)."""
    if len(out) != num_wg:
        return False
    seen = [False] * num_wg
    for t in out:
        t = int(t)
        if t < 0 or t >= num_wg or seen[t]:
            return False
        seen[t] = True
    return True


def xcd_tile_sets(out, num_xcd: int) -> list[list[int]]:
    """Tiles each XCD computes, in its dispatch order, under round-robin dispatch."""
    return [[int(out[w]) for w in bucket] for bucket in deal_round_robin(len(out), num_xcd)]


def fair_share(out, grid_m: int, grid_n: int, group_m: int, grouped: bool, num_xcd: int, renumbered: bool,
               skewed: bool = False) -> bool:
    """Every XCD works on its fair share of the raster, judged on the map itself.

    The tile count T comes from the grid, never from len(out).  XCD x (the workgroups w with
    w mod X == x) must hold T div X distinct raster positions, one more if x < T mod X; the shares of
    different XCDs must not overlap and together they must be the whole raster.  For a renumbering
    map (renumbered=True) XCD x's share must moreover begin right where the shares of XCDs 0..x-1
    end ("all contiguous blocks on the same XCD before moving to the next XCD").
    A map of the wrong length, a tile outside the grid, a tile handed out twice, or an XCD that
    holds a position of another XCD's share all fail.
    """
    total = grid_m * grid_n
    order = raster_order(grid_m, grid_n, group_m, grouped, skewed)
    pos = {pm * grid_n + pn: l for l, (pm, pn) in enumerate(order)}
    if len(out) != total:
        return False
    claimed: set[int] = set()
    begin = 0                                   # where XCD x's share begins if shares are laid end to end
    for x in range(num_xcd):
        want = total // num_xcd + (1 if x < total % num_xcd else 0)
        share = set()
        for w in range(x, len(out), num_xcd):
            t = int(out[w])
            if t not in pos:
                return False
            share.add(pos[t])
        if len(share) != want or share & claimed:
            return False
        if renumbered and want > 0 and min(share) != begin:
            return False
        claimed |= share
        begin += want
    return len(claimed) == total


def xcd_runs_contiguous(out, grid_m: int, grid_n: int, group_m: int, grouped: bool, num_xcd: int,
                        skewed: bool = False) -> bool:
    """Each XCD's tiles are one contiguous, increasing run of the raster order, runs abutting in XCD order."""
    order = raster_order(grid_m, grid_n, group_m, grouped, skewed)
    pos = {pm * grid_n + pn: l for l, (pm, pn) in enumerate(order)}
    expect = 0
    for tiles in xcd_tile_sets(out, num_xcd):
        for t in tiles:
            if pos[t] != expect:
                return False
            expect += 1
    return expect == len(out)
