"""The seeded input generators: determinism, ranges and the stated graph shapes (CPU)."""
import numpy as np
import torch

import synth


def test_mix64_matches_python_reference():
    x = torch.tensor([0, 1, 2, 12345678901234, -5], dtype=torch.int64)
    h = synth.mix64(x)
    for xi, hi in zip(x.tolist(), h.tolist()):
        assert (hi & ((1 << 64) - 1)) == synth.mix64_py(xi & ((1 << 64) - 1))


def test_streams_are_deterministic_and_sliceable():
    a = synth.normal(7, synth.S_FEAT, 100, 6)
    b = synth.normal_rows(7, synth.S_FEAT, 40, 60, 6)
    assert torch.equal(a[40:60], b)
    assert abs(a.mean().item()) < 0.15 and abs(a.std().item() - 1) < 0.15
    w = synth.glorot(7, 0, 30, 50)
    assert w.abs().max().item() <= (6 / 80) ** 0.5
    y = synth.labels(7, 1000, 16)
    assert y.min() >= 0 and y.max() < 16 and len(torch.unique(y)) == 16


def test_permutation_is_a_bijection():
    p = synth.permutation(3, synth.S_PERM_R, 1000)
    q = synth.permutation(3, synth.S_PERM_C, 1000)
    assert torch.equal(torch.sort(p).values, torch.arange(1000))
    assert not torch.equal(p, q)
    x = torch.arange(999)
    assert len(torch.unique(synth.affine_bijection(3, 2, 999, x))) == 999


def test_tiny_config_counts():
    c = synth.CONFIGS["tiny"]
    s, d = c.edges()
    assert s.numel() == 65536 and bool((s < d).all()) and int(d.max()) < c.n
    assert len(torch.unique(s * c.n + d)) == 65536
    s2, d2 = c.edges()
    assert torch.equal(s, s2) and torch.equal(d, d2)
    deg = torch.bincount(torch.cat([s, d]), minlength=c.n)
    assert deg.max().item() > 20 * deg.float().mean().item()       # power-law skew


def test_road_and_shard_shapes():
    c = synth.CONFIGS["road"].scaled(1e-3)
    s, d = c.edges()
    mean_deg = 2 * s.numel() / c.n
    assert 2.0 < mean_deg < 2.4
    sh = synth.CONFIGS["shard"].scaled(1e-3)
    rowptr, col, val = synth.shard_block(sh.seed, sh.m, sh.k, sh.n_samples)
    assert rowptr.numel() == sh.m + 1 and rowptr[-1].item() == col.numel() == val.numel()
    assert int(col.max()) < sh.k and float(val.min()) > 0
    for i in (0, 17, sh.m - 1):
        cs = col[rowptr[i]:rowptr[i + 1]]
        assert bool((cs[1:] > cs[:-1]).all())
