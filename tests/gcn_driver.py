"""Test helpers around the library's multi-layer sequencer."""
from __future__ import annotations

from typing import List

import numpy as np
import torch

import paper_2505_04083_amd as plx
from paper_2505_04083_amd.network import GcnNetwork


class NetworkRun:
    pass


def run_network(ctx, csr, H0: torch.Tensor, Ws: List[torch.Tensor], y: torch.Tensor, order=plx.PLX_ORDER_AUTO,
                backward: bool = True) -> NetworkRun:
    """Layer l uses orientation l % 2 (Eq. 5.3-5.4).  H0 is in P_c order; y in the order of the
    last layer's output.  Pre-activations are kept so that tests can compare every layer."""
    net = GcnNetwork(ctx, csr, Ws, dtype=H0.dtype, order=order, keep_preactivation=True)
    net.forward(H0)
    if backward:
        net.backward(H0, y)
    net.sync()
    run = NetworkRun()
    run.Z, run.F, run.dW, run.dF0, run.loss = net.Z, net.F, net.dW, net.dH[0], net.loss
    return run


def rel_err(gpu, ref: np.ndarray) -> float:
    """max |g - o| / max |o| over the whole tensor (the tolerance's definition)."""
    g = gpu.detach().double().cpu().numpy() if isinstance(gpu, torch.Tensor) else np.asarray(gpu, np.float64)
    denom = np.abs(ref).max()
    if denom == 0:
        return float(np.abs(g).max())
    return float(np.abs(g - ref).max() / denom)


def elt_err(gpu, ref: np.ndarray, floor: float = 1e-3) -> float:
    """Element-wise form of the tolerance: max over elements of |g - o| / max(|o|, floor * max |o|).  Unlike
    rel_err it weighs an error in a small entry (a low-degree row next to a hub) by that entry's own size,
    down to `floor` of the tensor's largest magnitude."""
    g = gpu.detach().double().cpu().numpy() if isinstance(gpu, torch.Tensor) else np.asarray(gpu, np.float64)
    top = np.abs(ref).max() if ref.size else 0.0
    if top == 0:
        return float(np.abs(g).max()) if g.size else 0.0
    return float((np.abs(g - ref) / np.maximum(np.abs(ref), floor * top)).max())
