"""Full-size parity in the launch configuration bench.py times: configs[3], one GPU's 7M x 28M
shard block (~200M stored entries), layer 32 -> 128, aggregate-first, only the activated output
stored.  The oracle cannot run the whole block in seconds, so it computes SAMPLED outputs one by
one (an output row of a sparse product depends only on its own CSR row) and the weight gradient
for a gradient whose support is the sampled rows (it is linear in the gradient)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_04083_amd as plx
import synth
from gcn_driver import rel_err

pytestmark = pytest.mark.gpu
TOL32 = 1e-4
DEV = "cuda:0"


@pytest.fixture(scope="module")
def shard():
    cfg = synth.CONFIGS["shard"]
    rowptr, col, val = synth.shard_block(cfg.seed, cfg.m, cfg.k, cfg.n_samples, DEV)
    X = synth.normal(cfg.seed, synth.S_FEAT, cfg.k, cfg.dims[0], DEV)
    W = synth.glorot(cfg.seed, 0, cfg.dims[0], cfg.dims[1], DEV)
    ctx = plx.plx_ctx(0)
    csr = plx.plx_csr_import(ctx, cfg.m, cfg.k, rowptr, col, val)
    host = dict(rowptr=rowptr.cpu().numpy(), col=col.cpu().numpy(), val=val.cpu().numpy(), X=X.cpu().numpy(),
                W=W.cpu().numpy().astype(np.float64))
    yield cfg, ctx, csr, X, W, host
    csr.close(); ctx.close()


def sample_rows(rowptr, n_long=600, n_empty=300, stride=9973):
    lens = np.diff(rowptr)
    m = len(lens)
    longest = np.argsort(lens)[-n_long:]
    empty = np.nonzero(lens == 0)[0][:n_empty]
    return np.unique(np.concatenate([np.arange(0, m, stride), longest, empty, [m - 1]])).astype(np.int64)


def test_shard_block_shape(shard):
    cfg, ctx, csr, X, W, h = shard
    assert abs(csr.nnz - 200e6) / 200e6 < 0.02            # ~200M stored entries, as the workload states
    (sub, wave, split), ent = plx.plx_csr_bins(csr, False)
    assert sub > 0 and wave > 0 and split > 0 and sum(ent) == csr.nnz     # all three kernels are exercised


def test_shard_forward_and_backward_samples(shard):
    cfg, ctx, csr, X, W, h = shard
    m, k, (din, dout) = cfg.m, cfg.k, cfg.dims
    S = sample_rows(h["rowptr"])
    order = plx.PLX_ORDER_AGG_FIRST
    ws = torch.empty(plx.plx_gcn_layer_workspace(csr, False, din, dout, order=order), dtype=torch.uint8, device=DEV)
    F = torch.empty(m, dout, device=DEV); saved = torch.empty(m, din, device=DEV)
    plx.plx_gcn_layer_fwd(ctx, csr, False, X, W, None, F, saved, ws, order=order)
    plx.plx_sync(ctx)
    # forward: Eq. 2.1 rows, then Eq. 2.2 + 2.3 on them
    Hs = oracle.spmm_rows_csr(h["rowptr"], h["col"], h["val"], h["X"], S)
    Qs = oracle.gemm(Hs, h["W"])
    Sd = torch.as_tensor(S, device=DEV)
    assert rel_err(saved[Sd], Hs) <= TOL32
    assert rel_err(F[Sd], oracle.relu(Qs)) <= TOL32
    assert bool((saved[Sd][torch.as_tensor(np.diff(h["rowptr"])[S] == 0, device=DEV)] == 0).all())

    # backward with a gradient supported on the sampled rows (rows whose mask decision is
    # ill-conditioned, |Q| < 1e-5, get a zero gradient so both sides take the same decision)
    r = np.random.default_rng(3)
    dFs = r.standard_normal((len(S), dout)).astype(np.float32)
    dFs[np.abs(Qs).min(axis=1) < 1e-5] = 0.0
    dF = torch.zeros(m, dout, device=DEV)
    dF[Sd] = torch.as_tensor(dFs, device=DEV)
    dX = torch.empty(k, din, device=DEV); dW = torch.empty(din, dout, device=DEV)
    plx.plx_gcn_layer_bwd(ctx, csr, False, X, W, F, dF, saved, dX, dW, ws, order=order)
    plx.plx_sync(ctx)
    dQ = oracle.relu_bwd(Qs, dFs)                                   # Eq. 2.4
    assert rel_err(dW, oracle.gemm(Hs, dQ, ta=True)) <= TOL32       # Eq. 2.5 (other rows contribute 0)
    dS = np.zeros((m, din)); dS[S] = oracle.gemm(dQ, h["W"], tb=True)   # Eq. 2.6
    # Eq. 2.7 on sampled output rows: columns met by sampled rows, plus a stride of others
    cols_hit = np.unique(np.concatenate([h["col"][h["rowptr"][i]:h["rowptr"][i + 1]] for i in S[::7]]))
    J = np.unique(np.concatenate([cols_hit[:: max(1, len(cols_hit) // 3000)], np.arange(0, k, 99991)])).astype(np.int64)
    ref = oracle.spmm_t_rows_csr(m, k, h["rowptr"], h["col"], h["val"], dS, J)
    assert np.abs(ref).max() > 0
    assert rel_err(dX[torch.as_tensor(J, device=DEV)], ref) <= TOL32


def test_shard_backward_dense_gradient_samples(shard):
    """The benchmark's own inputs (dense random gradient): sampled rows of dX through the whole
    chain Eq. 2.1 -> 2.2 -> 2.4 -> 2.6 -> 2.7, the oracle evaluating exactly the rows it needs."""
    cfg, ctx, csr, X, W, h = shard
    m, k, (din, dout) = cfg.m, cfg.k, cfg.dims
    order = plx.PLX_ORDER_AGG_FIRST
    dF = synth.normal(cfg.seed, synth.S_AUX, m, dout, DEV)
    ws = torch.empty(plx.plx_gcn_layer_workspace(csr, False, din, dout, order=order), dtype=torch.uint8, device=DEV)
    F = torch.empty(m, dout, device=DEV); saved = torch.empty(m, din, device=DEV)
    dX = torch.empty(k, din, device=DEV); dW = torch.empty(din, dout, device=DEV)
    plx.plx_gcn_layer_fwd(ctx, csr, False, X, W, None, F, saved, ws, order=order)
    plx.plx_gcn_layer_bwd(ctx, csr, False, X, W, F, dF, saved, dX, dW, ws, order=order)
    plx.plx_sync(ctx)
    # sampled output rows j of dX and the block rows i that touch them
    J = np.arange(17, k, 70001, dtype=np.int64)
    rowptr, col = h["rowptr"], h["col"]
    hit = np.nonzero(np.isin(col, J))[0]
    rows_needed = np.unique(np.searchsorted(rowptr, hit, side="right") - 1).astype(np.int64)
    assert 0 < len(rows_needed) < 200000
    Hn = oracle.spmm_rows_csr(rowptr, col, h["val"], h["X"], rows_needed)
    Qn = oracle.gemm(Hn, h["W"])
    dFn = dF[torch.as_tensor(rows_needed, device=DEV)].cpu().numpy()
    dSn = oracle.gemm(oracle.relu_bwd(Qn, dFn), h["W"], tb=True)
    dS = np.zeros((m, din)); dS[rows_needed] = dSn
    ref = oracle.spmm_t_rows_csr(m, k, rowptr, col, h["val"], dS, J)
    # rows j fed by a row whose mask decision is ill-conditioned are left out of the comparison
    shaky = rows_needed[np.abs(Qn).min(axis=1) < 1e-5]
    if len(shaky):
        bad_cols = np.unique(np.concatenate([col[rowptr[i]:rowptr[i + 1]] for i in shaky]))
        keep = ~np.isin(J, bad_cols)
        J, ref = J[keep], ref[keep]
    assert len(J) > 100
    assert rel_err(dX[torch.as_tensor(J, device=DEV)], ref) <= TOL32
