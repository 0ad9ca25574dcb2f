"""The block-balance statistic of the studies (Table 3) on GPU-built matrices against the oracle's."""
import numpy as np
import pytest
import torch

import oracle
from oracle import dense as odense
import paper_2505_04083_amd as plx
import studies
import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_block_balance_of_gpu_built_matrices_matches_the_oracle():
    """studies.block_ratio (max / mean entry count over an 8 x 8 tiling of the matrix plx_build_csr stores) equals
    oracle.dense.block_balance of the same matrix built by the oracle, for the original order, a single permutation
    (P A P^T, Eq. 5.1-5.2) and the double permutation (P_r A P_c^T, Eq. 5.3); the single permutation also equals
    the closed form behind Table 3's 3.24 (the N self-loops stay on the 8 diagonal blocks) to sampling noise, and
    the double permutation is balanced."""
    cfg = synth.CONFIGS["road"].scaled(4e-3)                  # 200,000 nodes, the road recipe
    src, dst = cfg.edges()
    pr, pc = cfg.perms()
    adj = oracle.adjacency(cfg.n, src.numpy(), dst.numpy())
    ctx = plx.plx_ctx(0)
    got, want = {}, {}
    for name, (a, b) in {"original": (None, None), "single": (pr, pr), "double": (pr, pc)}.items():
        csr = plx.plx_build_csr(ctx, cfg.n, src.to(DEV), dst.to(DEV), None if a is None else a.to(DEV),
                                None if b is None else b.to(DEV))
        got[name] = studies.block_ratio(ctx, csr, cfg.n, 8)
        r = adj.row if a is None else a.numpy()[adj.row]
        c = adj.col if b is None else b.numpy()[adj.col]
        want[name] = odense.block_balance(cfg.n, r, c, 8)
        nnz = csr.nnz
        csr.close()
        assert abs(got[name] - want[name]) <= 1e-12 * want[name], (name, got[name], want[name])
    closed = ((nnz - cfg.n) / 64 + cfg.n / 8) / (nnz / 64)
    assert abs(got["single"] - closed) / closed < 0.02
    assert got["double"] < 1.05 < got["single"] < got["original"]
    ctx.close()
