"""Dense brute force for tiny graphs, numpy fp64 -- TEST INFRASTRUCTURE.

Second, independent form of the oracle: the normalised adjacency is materialised as an
N x N array straight from the edge list (Sec. 2.1) and the network is evaluated with numpy
matrix products.  Nothing here calls the C loops, so agreement between the two forms pins
both.  Also holds the block-balance statistic of Table 3.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


def dense_adjacency(n: int, src, dst) -> Tuple[np.ndarray, np.ndarray]:
    """(A^ as n x n fp64, degrees): self-loops added, then D^-1/2 (A+I) D^-1/2 (Sec. 2.1)."""
    A = np.zeros((n, n), np.float64)
    for u, v in zip(np.asarray(src).tolist(), np.asarray(dst).tolist()):
        if u != v:
            A[u, v] = 1.0
            A[v, u] = 1.0
    A[np.arange(n), np.arange(n)] = 1.0
    d = A.sum(axis=1)
    s = 1.0 / np.sqrt(d)
    return s[:, None] * A * s[None, :], d.astype(np.int64)


def permutation_matrix(perm) -> np.ndarray:
    """P with P[perm[i], i] = 1, so (P x)[perm[i]] = x[i]: perm sends an original id to its new id (Sec. 5.1)."""
    perm = np.asarray(perm)
    n = perm.shape[0]
    P = np.zeros((n, n), np.float64)
    P[perm, np.arange(n)] = 1.0
    return P


def gcn_forward_backward(A: np.ndarray, F0, Ws: Sequence, y):
    """Returns (logits, loss, [dW_l], dF0) with numpy products; same equations as oracle.gcn."""
    F = np.asarray(F0, np.float64)
    n = F.shape[0]
    Hs, Qs = [], []
    L = len(Ws)
    for l, W in enumerate(Ws):
        H = A @ F
        Q = H @ np.asarray(W, np.float64)
        Hs.append(H); Qs.append(Q)
        if l + 1 < L:
            F = np.maximum(Q, 0.0)
    Z = Qs[-1]
    e = np.exp(Z - Z.max(axis=1, keepdims=True))
    p = e / e.sum(axis=1, keepdims=True)
    y = np.asarray(y)
    loss = float(-np.log(p[np.arange(n), y]).mean())
    dQ = p.copy()
    dQ[np.arange(n), y] -= 1.0
    dQ /= n
    dWs = [None] * L
    dF = None
    for l in range(L - 1, -1, -1):
        if l + 1 < L:
            dQ = dF * (Qs[l] > 0.0)
        dWs[l] = Hs[l].T @ dQ
        dF = A.T @ (dQ @ np.asarray(Ws[l], np.float64).T)
    return Z, loss, dWs, dF


def block_balance(n: int, row, col, blocks: int) -> float:
    """Table 3's statistic: max / mean of the nonzero counts over a blocks x blocks tiling of
    an n x n matrix whose nonzeros are (row[e], col[e])."""
    row, col = np.asarray(row, np.int64), np.asarray(col, np.int64)
    edges = (np.arange(blocks + 1, dtype=np.int64) * n) // blocks
    bi = np.searchsorted(edges, row, side="right") - 1
    bj = np.searchsorted(edges, col, side="right") - 1
    cnt = np.bincount(bi * blocks + bj, minlength=blocks * blocks)
    return float(cnt.max() / cnt.mean())
