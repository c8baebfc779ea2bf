"""Reference transpose (test infrastructure only): out[j][i] = in[i][j], elements moved verbatim.

The paper's transpose case study (SwizzlePerf, Results; Appendix "Case Study: Other Swizzling
Pattern Examples") changes which workgroup moves which tile, never the result, so the oracle is
the definition itself: two loops for small inputs, numpy's transpose for large ones.
"""
from __future__ import annotations

import numpy as np


def transpose_loops(x) -> list[list[int]]:
    rows, cols = len(x), len(x[0])
    out = [[0] * rows for _ in range(cols)]
    for i in range(rows):
        for j in range(cols):
            out[j][i] = x[i][j]
    return out


def transpose(x: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x).T)
