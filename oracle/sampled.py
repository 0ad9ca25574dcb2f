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


def adjacency_rows(n: int, src: np.ndarray, dst: np.ndarray, deg: np.ndarray,
                   nodes: np.ndarray) -> Dict[int, Tuple[np.ndarray, np.ndarray]]:
    """{u: (neighbour ids incl. u itself, ascending; values 1/sqrt(d_u d_v) in fp64)}: rows u of A^ in ORIGINAL ids."""
    nodes = np.asarray(nodes, np.int64)
    slot = np.full(n, -1, np.int64)
    slot[nodes] = np.arange(len(nodes))
    nbrs = [[int(u)] for u in nodes]
    for a, b in ((src, dst), (dst, src)):
        hit = np.nonzero(slot[a] >= 0)[0]
        for s, v in zip(slot[a[hit]].tolist(), b[hit].tolist()):
            nbrs[s].append(v)
    out = {}
    for u, vs in zip(nodes.tolist(), nbrs):
        vs = np.sort(np.asarray(vs, np.int64))
        out[int(u)] = (vs, 1.0 / np.sqrt(float(deg[u]) * deg[vs].astype(np.float64)))
    return out


class Block:
    """The sub-matrix A^[rows, cols] as a coordinate list in positions (row position ascending): every neighbour of a
    node of `rows` must be in `cols` (the block is then the whole of those rows)."""

    def __init__(self, rows_of: Dict[int, Tuple[np.ndarray, np.ndarray]], rows: np.ndarray, cols: np.ndarray):
        cols = np.asarray(cols, np.int64)                      # ascending, unique
        r, c, v = [], [], []
        for i, u in enumerate(np.asarray(rows, np.int64).tolist()):
            ids, vals = rows_of[u]
            pos = np.searchsorted(cols, ids)
            if not np.array_equal(cols[np.minimum(pos, len(cols) - 1)], ids):
                raise ValueError("column set does not cover the neighbours of the row set")
            r.append(np.full(len(ids), i, np.int64)); c.append(pos.astype(np.int64)); v.append(vals)
        self.m, self.k = len(rows), len(cols)
        self.row = np.concatenate(r) if r else np.zeros(0, np.int64)
        self.col = np.concatenate(c) if c else np.zeros(0, np.int64)
        self.val = np.concatenate(v) if v else np.zeros(0, np.float64)


def receptive_field(n: int, src: np.ndarray, dst: np.ndarray, deg: np.ndarray, nodes: np.ndarray, hops: int):
    """[V_0 = nodes (sorted, unique), V_1, ..., V_hops] with V_{h+1} = V_h and all its neighbours, and the rows of A^ for
    every node of V_{hops-1}."""
    V = [np.unique(np.asarray(nodes, np.int64))]
    rows_of: Dict[int, Tuple[np.ndarray, np.ndarray]] = {}
    for _ in range(hops):
        new = np.array([u for u in V[-1].tolist() if u not in rows_of], np.int64)
        rows_of.update(adjacency_rows(n, src, dst, deg, new))
        V.append(np.unique(np.concatenate([rows_of[int(u)][0] for u in V[-1].tolist()] + [V[-1]])))
    return V, rows_of


def network_on_samples(n, src, dst, deg, F0_rows, Ws, nodes, dQ_last):
    """An L-layer GCN (Eq. 2.1-2.3) evaluated only where the outputs at `nodes` need it, and its backward pass
    (Eq. 2.4-2.7) for a loss gradient dQ_last given on `nodes` and zero on every other node.

    F0_rows(ids) returns the input features of the given original node ids.  With V_0 = nodes and V_h its h-hop
    closure, layer l needs its input on V_{L-l} and gives its output on V_{L-l-1}; each step is one of this
    package's plain loops on the block A^[V_{h-1}, V_h].  Returns (V, logits on V_0, [dW_l], dF0 on V_L, Q: list of
    the pre-activations Q_l on V_{L-l-1}).  Rows of dF0 outside V_L are exactly zero."""
    from . import gemm, relu, relu_bwd, spmm_coo, spmm_t_coo
    L = len(Ws)
    V, rows_of = receptive_field(n, src, dst, deg, nodes, L)
    blocks = [Block(rows_of, V[L - l - 1], V[L - l]) for l in range(L)]       # block of layer l
    F = np.asarray(F0_rows(V[L]), np.float64)
    H, Q = [], []
    for l, W in enumerate(Ws):
        b = blocks[l]
        H.append(spmm_coo(b.m, b.row, b.col, b.val, F))                       # Eq. 2.1
        Q.append(gemm(H[l], np.asarray(W, np.float64)))                       # Eq. 2.2
        if l + 1 < L:
            F = relu(Q[l])                                                    # Eq. 2.3
    dQ = np.asarray(dQ_last, np.float64)
    dW = [None] * L
    dF = None
    for l in range(L - 1, -1, -1):
        b = blocks[l]
        if l + 1 < L:
            dQ = relu_bwd(Q[l], dF)                                           # Eq. 2.4
        dW[l] = gemm(H[l], dQ, ta=True)                                       # Eq. 2.5 (rows outside V carry a zero dQ)
        dH = gemm(dQ, np.asarray(Ws[l], np.float64), tb=True)                 # Eq. 2.6
        dF = spmm_t_coo(b.k, b.row, b.col, b.val, dH)                         # Eq. 2.7
    return V, Q[-1], dW, dF, Q
