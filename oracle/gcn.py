"""L-layer GCN forward + backward on the UNPERMUTED graph, in fp64 -- TEST INFRASTRUCTURE.

Follows the paper's notation (Sec. 2.1): layer input F, aggregation H = A^ F (Eq. 2.1),
combination Q = H W (Eq. 2.2), activation F' = ReLU(Q) (Eq. 2.3, not applied after the last
layer, whose Q are the logits), and backward dQ = dF' * ReLU'(Q) (Eq. 2.4), dW = H^T dQ
(Eq. 2.5), dH = dQ W^T (Eq. 2.6), dF = A^^T dH (Eq. 2.7), computed for layer 0 as well
(the input features are trainable).  Every step calls the plain C loops of this package.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence

import numpy as np

from . import Adjacency, gemm, relu, relu_bwd, softmax_ce, spmm_coo, spmm_t_coo


@dataclass
class Trace:
    F: List[np.ndarray] = field(default_factory=list)    # F[l] input of layer l (F[0] = features)
    H: List[np.ndarray] = field(default_factory=list)    # H[l] = A^ F[l]
    Q: List[np.ndarray] = field(default_factory=list)    # Q[l] = H[l] W[l]
    loss: float = 0.0
    dQ: List[np.ndarray] = field(default_factory=list)
    dW: List[np.ndarray] = field(default_factory=list)
    dH: List[np.ndarray] = field(default_factory=list)
    dF: List[np.ndarray] = field(default_factory=list)   # dF[l] = gradient wrt F[l]

    @property
    def logits(self) -> np.ndarray:
        return self.Q[-1]


def forward(adj: Adjacency, F0, Ws: Sequence) -> Trace:
    t = Trace()
    F = np.asarray(F0, np.float64)
    L = len(Ws)
    for l, W in enumerate(Ws):
        t.F.append(F)
        H = spmm_coo(adj.n, adj.row, adj.col, adj.val, F)          # Eq. 2.1
        Q = gemm(H, np.asarray(W, np.float64))                     # Eq. 2.2
        t.H.append(H); t.Q.append(Q)
        if l + 1 < L:
            F = relu(Q)                                            # Eq. 2.3
    return t


def forward_backward(adj: Adjacency, F0, Ws: Sequence, y) -> Trace:
    t = forward(adj, F0, Ws)
    L = len(Ws)
    t.loss, dQ = softmax_ce(t.Q[-1], y)
    t.dQ = [None] * L; t.dW = [None] * L; t.dH = [None] * L; t.dF = [None] * L
    for l in range(L - 1, -1, -1):
        if l + 1 < L:
            dQ = relu_bwd(t.Q[l], t.dF[l + 1])                     # Eq. 2.4
        t.dQ[l] = dQ
        t.dW[l] = gemm(t.H[l], dQ, ta=True)                        # Eq. 2.5
        t.dH[l] = gemm(dQ, np.asarray(Ws[l], np.float64), tb=True)  # Eq. 2.6
        t.dF[l] = spmm_t_coo(adj.n, adj.row, adj.col, adj.val, t.dH[l])   # Eq. 2.7
    return t


def loss_only(adj: Adjacency, F0, Ws: Sequence, y) -> float:
    t = forward(adj, F0, Ws)
    return softmax_ce(t.Q[-1], y)[0]
