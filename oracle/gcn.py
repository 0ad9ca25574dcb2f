"""L-layer GCN forward + backward on the UNPERMUTED graph, in fp64 -- TEST INFRASTRUCTURE.

Follows the paper's notation (Sec. 2.1): layer input F, aggregation H = A^ F (Eq. 2.1),
combination Q = H W (Eq. 2.2), activation F' = ReLU(Q) (Eq. 2.3, not applied after the last
layer, whose Q are the logits), and backward dQ = dF' * ReLU'(Q) (Eq. 2.4), dW = H^T dQ
(Eq. 2.5), dH = dQ W^T (Eq. 2.6), dF = A^^T dH (Eq. 2.7), computed for layer 0 as well
(the input features are trainable).  Every step calls the plain C loops of this package.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

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


def backward_from(adj: Adjacency, t: Trace, Ws: Sequence, dQ_last, masks: Optional[Sequence] = None) -> Trace:
    """Eq. 2.4-2.7 for every layer, starting from the gradient dQ_last with respect to the last layer's Q.

    masks (optional): masks[l] is a 0/1 array that takes the place of [Q_l > 0] in Eq. 2.4.  The sign of Q_l is an
    integer decision; when the implementation under test stores its activations in a narrower type, that decision is
    taken in ITS precision and handed in here, so that both sides differentiate the same piecewise-linear function."""
    L = len(Ws)
    dQ = np.asarray(dQ_last, np.float64)
    t.dQ = [None] * L; t.dW = [None] * L; t.dH = [None] * L; t.dF = [None] * L
    for l in range(L - 1, -1, -1):
        if l + 1 < L:
            if masks is not None and masks[l] is not None:
                dQ = t.dF[l + 1] * np.asarray(masks[l], np.float64)  # Eq. 2.4, decision given
            else:
                dQ = relu_bwd(t.Q[l], t.dF[l + 1])                 # Eq. 2.4
        t.dQ[l] = dQ
        t.dW[l] = gemm(t.H[l], dQ, ta=True)                        # Eq. 2.5
        t.dH[l] = gemm(dQ, np.asarray(Ws[l], np.float64), tb=True)  # Eq. 2.6
        t.dF[l] = spmm_t_coo(adj.n, adj.row, adj.col, adj.val, t.dH[l])   # Eq. 2.7
    return t


def forward_backward(adj: Adjacency, F0, Ws: Sequence, y, masks: Optional[Sequence] = None) -> Trace:
    t = forward(adj, F0, Ws)
    t.loss, dQ = softmax_ce(t.Q[-1], y)
    return backward_from(adj, t, Ws, dQ, masks)


def loss_only(adj: Adjacency, F0, Ws: Sequence, y) -> float:
    t = forward(adj, F0, Ws)
    return softmax_ce(t.Q[-1], y)[0]
