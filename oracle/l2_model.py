"""Lock-step panel-count model of per-XCD L2 reuse (test / harness infrastructure only).

The paper's argument (SwizzlePerf, Appendix "Case Study: GEMM Swizzling"): tiles in one row
of C read the same rows of A, tiles in one column of C read the same columns of B, so the
tiles that share an XCD's L2 should share rows and columns.  This model counts exactly that.
Assumptions: workgroup w runs on XCD w mod X; an XCD runs `slots` tiles at a time, in
dispatch order, and those advance through K together.  Per batch of co-resident tiles every
tile asks for one A panel and one B panel; a panel already asked for by a co-resident tile
is a hit.  Predicted hit rate = 1 - distinct panels / requested panels.

It predicts the sign and rough size of the effect of a PID map; it is not a cache simulator.
"""
from __future__ import annotations

from .pid_map import deal_round_robin


def predicted_hit_rate(out, grid_n: int, num_xcd: int, slots: int) -> float:
    requested = 0
    distinct = 0
    for bucket in deal_round_robin(len(out), num_xcd):
        for s in range(0, len(bucket), slots):
            batch = [int(out[w]) for w in bucket[s:s + slots]]
            rows = {t // grid_n for t in batch}
            cols = {t % grid_n for t in batch}
            requested += 2 * len(batch)
            distinct += len(rows) + len(cols)
    return 1.0 - distinct / requested if requested else 0.0
