"""L-layer GCN forward + backward as a fixed sequence of C-ABI calls (no arithmetic here).

Layer l uses the stored orientation l % 2 (Eq. 5.3-5.4 of the paper: P_r A P_c^T for even layers,
P_c A P_r^T for odd ones).  All buffers are allocated once, so a training step allocates nothing.
Hidden layers store only the activated output (its sign serves Eq. 2.4) and, where the dense product
of the layer can write them on the fly (aggregate-first order, widths up to 128), that sign packed
one bit per element, which is all the backward pass then reads of it; the last layer stores the
logits.  Where a combine-first layer follows an aggregate-first one of fitting widths, the gradient
matrix between them is never formed: the later layer's backward call stops at dT = A^T dZ and the
earlier one takes (dT, W) in its place; in the forward pass the earlier layer's last product also
forms the later layer's T = F W, so F is written for the backward pass but not read back (`chain`).  The input must be in P_c order and the labels in the order of the last layer's output."""
from __future__ import annotations

from typing import List, Optional

import torch

from . import (PLX_ACT_NONE, PLX_ACT_RELU, PLX_ACT_RELU_BITS, PLX_BF16, PLX_F32, PLX_ORDER_AUTO, plx_gcn_layer_bwd,
               plx_gcn_layer_bwd_chained, plx_gcn_layer_bwd_chained_workspace, plx_gcn_layer_bwd_dt, plx_gcn_layer_fwd,
               plx_gcn_layer_fwd_chained, plx_gcn_layer_fwd_from_t, plx_gcn_layer_plan, plx_gcn_layer_workspace, plx_softmax_ce, plx_sync)


def aligned_rows(rows: int, cols: int, dtype, dev) -> torch.Tensor:
    """rows x cols view with 16-byte aligned rows (128-bit row accesses in the sparse and the dense kernels): the
    layout every matrix of the network is kept in.  Rows shorter than 256 bytes get a pitch of a multiple of 64
    bytes, so that a gathered row never touches a cache line more than it must (measured: -0.5 to -2 % per step on
    the graph workloads whose narrowest width is 41, 47 or 100 elements)."""
    es = 4 if dtype == torch.float32 else 2
    pitch = 64 if cols * es < 256 else 16            # bytes
    q = pitch // es
    ld = (cols + q - 1) // q * q
    return torch.empty(rows, ld, dtype=dtype, device=dev)[:, :cols]


class GcnNetwork:
    def __init__(self, ctx, csr, Ws: List[torch.Tensor], dtype=torch.float32, order: int = PLX_ORDER_AUTO,
                 keep_preactivation: bool = False, sign_bits: bool = True, chain: bool = True, input_grad: bool = True):
        """input_grad=False: the gradient with respect to the network's input features (Eq. 2.6-2.7 of the first layer,
        which no weight update needs) is not formed; dH[0] is then None and every dW is unchanged."""
        self.ctx, self.csr, self.Ws, self.order = ctx, csr, Ws, order
        self.L = len(Ws)
        dev = Ws[0].device
        code = PLX_F32 if dtype == torch.float32 else PLX_BF16
        self.act = [PLX_ACT_RELU if l + 1 < self.L else PLX_ACT_NONE for l in range(self.L)]
        # Which layers keep their ReLU mask as sign bits, and which consecutive pairs are chained, is the library's answer
        # (plx_gcn_layer_plan): the shape limits of the kernels are stated in one place, the C side.
        #   chained[l]: layer l+1 (combine-first) hands layer l its dT and W instead of the gradient matrix between them,
        #     which layer l's fused backward kernel then forms tile by tile (road graph, 64-128-16, 50 M nodes: the step costs
        #     layer l's kernel 3 % and saves layer l+1's kernel the 25.6 GB write of the gradient, 10.5 -> 4.9 ms);
        #   fwd_chained[l]: the product that writes layer l's output also forms T = F W of layer l+1, which then starts
        #     from T instead of reading F back.
        agg = []
        self.chained = [False] * self.L
        self.fwd_chained = [False] * self.L
        for l, W in enumerate(Ws):
            din, dout = W.shape
            last = l + 1 == self.L
            dn = 0 if (last or not chain) else Ws[l + 1].shape[1]
            a, bits, cf, cb = plx_gcn_layer_plan(ctx, din, dout, dn, code, order, order,
                                                 keep_values=keep_preactivation or not sign_bits or last)
            agg.append(a)
            if bits and not last:
                self.act[l] = PLX_ACT_RELU_BITS
            self.chained[l], self.fwd_chained[l] = cb, cf
        nbytes = 1
        for l, W in enumerate(Ws):
            if self.chained[l]:
                need = plx_gcn_layer_bwd_chained_workspace(ctx, csr, bool(l % 2), W.shape[0], W.shape[1], Ws[l + 1].shape[1], code,
                                                           self.act[l], order)
            else:
                need = plx_gcn_layer_workspace(csr, bool(l % 2), W.shape[0], W.shape[1], code, self.act[l], order)
            nbytes = max(nbytes, need)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        self.Z: List[Optional[torch.Tensor]] = []
        self.F: List[Optional[torch.Tensor]] = []
        self.saved: List[torch.Tensor] = []
        self.dH: List[Optional[torch.Tensor]] = []
        self.dT: List[Optional[torch.Tensor]] = []
        self.T: List[Optional[torch.Tensor]] = []               # T[l] = F[l-1] W[l], written by layer l-1's forward call
        self.dW: List[torch.Tensor] = []
        for l, W in enumerate(Ws):
            rows, cols = csr.shape(bool(l % 2))
            din, dout = W.shape
            last = l + 1 == self.L
            if self.act[l] == PLX_ACT_RELU_BITS:
                self.Z.append(torch.empty(rows, (dout + 31) // 32, dtype=torch.int32, device=dev))
            else:
                self.Z.append(aligned_rows(rows, dout, dtype, dev) if (last or keep_preactivation) else None)
            self.F.append(None if last else aligned_rows(rows, dout, dtype, dev))
            self.saved.append(aligned_rows(rows if agg[l] else 1, din, dtype, dev))
            hands_dt = l > 0 and self.chained[l - 1]             # then dH[l] is never formed: dT[l] goes to layer l-1
            self.dH.append(None if (hands_dt or (l == 0 and not input_grad)) else aligned_rows(cols, din, dtype, dev))
            self.dT.append(aligned_rows(cols, dout, dtype, dev) if hands_dt else None)
            self.T.append(aligned_rows(cols, dout, dtype, dev) if (l > 0 and self.fwd_chained[l - 1]) else None)
            self.dW.append(torch.empty(din, dout, dtype=torch.float32, device=dev))
        rows_last = csr.shape(bool((self.L - 1) % 2))[0]
        self.dZ_last = aligned_rows(rows_last, Ws[-1].shape[1], dtype, dev)
        self.row_loss = torch.empty(max(1, rows_last), dtype=torch.float32, device=dev)
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)

    def forward(self, H0: torch.Tensor) -> torch.Tensor:
        h = H0
        for l, W in enumerate(self.Ws):
            if l > 0 and self.fwd_chained[l - 1]:                # T of this layer came out of the previous call
                plx_gcn_layer_fwd_from_t(self.ctx, self.csr, bool(l % 2), self.T[l], self.Z[l], self.F[l], act=self.act[l])
            elif l + 1 < self.L and self.fwd_chained[l]:
                plx_gcn_layer_fwd_chained(self.ctx, self.csr, bool(l % 2), h, W, self.Z[l], self.F[l], self.saved[l],
                                          self.Ws[l + 1], self.T[l + 1], self.ws, act=self.act[l], order=self.order)
            else:
                plx_gcn_layer_fwd(self.ctx, self.csr, bool(l % 2), h, W, self.Z[l], self.F[l], self.saved[l], self.ws,
                                  act=self.act[l], order=self.order)
            if l + 1 < self.L:
                h = self.F[l]
        return self.Z[-1]

    def backward(self, H0: torch.Tensor, y: torch.Tensor) -> None:
        plx_softmax_ce(self.ctx, self.Z[-1], y, self.dZ_last, row_loss=self.row_loss, loss=self.loss)
        self.backward_from(H0, self.dZ_last)

    def backward_from(self, H0: torch.Tensor, grad: torch.Tensor) -> None:
        """The backward calls of every layer for a given gradient with respect to the last layer's output."""
        for l in range(self.L - 1, -1, -1):
            h = H0 if l == 0 else self.F[l - 1]
            mask_src = None if self.act[l] == PLX_ACT_NONE else (self.Z[l] if self.Z[l] is not None else self.F[l])
            if l + 1 < self.L and self.chained[l]:               # grad is the dT of layer l+1
                plx_gcn_layer_bwd_chained(self.ctx, self.csr, bool(l % 2), h, self.Ws[l], mask_src, grad, self.Ws[l + 1],
                                          self.saved[l], self.dH[l], self.dW[l], self.ws, act=self.act[l], order=self.order)
                grad = self.dH[l]
            elif l > 0 and self.chained[l - 1]:                  # stops at dT; layer l-1 forms its dF from (dT, W)
                plx_gcn_layer_bwd_dt(self.ctx, self.csr, bool(l % 2), h, mask_src, grad, self.dT[l], self.dW[l], self.ws,
                                     act=self.act[l])
                grad = self.dT[l]
            else:
                plx_gcn_layer_bwd(self.ctx, self.csr, bool(l % 2), h, self.Ws[l], mask_src, grad, self.saved[l],
                                  self.dH[l], self.dW[l], self.ws, act=self.act[l], order=self.order)
                grad = self.dH[l]

    def step(self, H0: torch.Tensor, y: torch.Tensor) -> None:
        self.forward(H0)
        self.backward(H0, y)

    def sync(self) -> None:
        plx_sync(self.ctx)

    def capture(self, H0: torch.Tensor, y: torch.Tensor, stream: torch.cuda.Stream) -> "torch.cuda.CUDAGraph":
        """Record one forward + backward into a HIP graph (for small, launch-bound graphs the ~30
        launches of a step then cost one graph launch).  `stream` must be the non-default stream the
        context was created on.  A step allocates nothing and never waits (every buffer belongs to
        this object, to the adjacency handle or to the workspace), so it can be recorded as it is.
        Per-kernel timing must be off."""
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream, capture_error_mode="thread_local"):
            self.step(H0, y)
        return graph
