"""Single rows of the normalised, double-permuted adjacency straight from the definition, for
graphs too large to build whole on the host -- TEST INFRASTRUCTURE.

Row u of A^ = D^-1/2 (A + I) D^-1/2 (paper Sec. 2.1) needs only u's distinct neighbours and the
degrees d = (number of distinct neighbours) + 1; row perm_r[u] of P_r A^ P_c^T (Eq. 5.3) is the same
entries with columns relabelled by perm_c and sorted.  Precondition (the generators' contract,
checked by the caller): the edge list holds every undirected edge exactly once and no loops, so
degrees are plain counts.
"""
from __future__ import annotations

from typing import Dict, Tuple

import numpy as np


def degrees(n: int, src: np.ndarray, dst: np.ndarray) -> np.ndarray:
    """d_u = 1 + number of edges touching u (distinct-edge, loop-free list)."""
    return 1 + np.bincount(src, minlength=n) + np.bincount(dst, minlength=n)


def permuted_rows(n: int, src: np.ndarray, dst: np.ndarray, deg: np.ndarray, perm_r: np.ndarray,
                  perm_c: np.ndarray, nodes: np.ndarray) -> Dict[int, Tuple[np.ndarray, np.ndarray]]:
    """{perm_r[u]: (columns int32 ascending, values float32)} for every u in `nodes`."""
    nodes = np.asarray(nodes, np.int64)
    slot = np.full(n, -1, np.int64)
    slot[nodes] = np.arange(len(nodes))
    nbrs = [[int(u)] for u in nodes]                     # the self-loop
    for a, b in ((src, dst), (dst, src)):
        hit = np.nonzero(slot[a] >= 0)[0]
        for s, v in zip(slot[a[hit]].tolist(), b[hit].tolist()):
            nbrs[s].append(v)
    out = {}
    for u, vs in zip(nodes.tolist(), nbrs):
        vs = np.asarray(vs, np.int64)
        cols = perm_c[vs]
        order = np.argsort(cols)
        vals = (1.0 / np.sqrt(float(deg[u]) * deg[vs].astype(np.float64))).astype(np.float32)
        out[int(perm_r[u])] = (cols[order].astype(np.int32), vals[order])
    return out
