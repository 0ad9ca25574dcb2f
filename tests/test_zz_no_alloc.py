"""The allocation-free sparse product (plx_spmm_static) against plx_spmm / plx_spmm_t and the oracle.

Collected last (file name): it shares one fixed per-GPU buffer between all its calls, and runs two calls
in a row, the second on a smaller input, so that stale partial sums of the first would show."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_04083_amd as plx
from gcn_driver import elt_err, rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def block(m, k, seed, long_rows):
    """CSR block with skewed row lengths, empty rows, and `long_rows` rows of 256+ entries (the rows whose
    partial sums go through the buffer under test), one of them far beyond the segment length."""
    r = np.random.default_rng(seed)
    lens = np.minimum(r.zipf(1.7, m), 200).astype(np.int64)
    lens[r.integers(0, m, m // 9)] = 0
    pick = r.choice(m, long_rows, replace=False)
    lens[pick] = r.integers(256, min(k, 3000), long_rows)
    lens[pick[0]] = min(k, 9000)
    rowptr = np.zeros(m + 1, np.int64); rowptr[1:] = np.cumsum(lens)
    col = np.concatenate([np.sort(r.choice(k, l, replace=False)) for l in lens if l > 0])
    val = (r.random(len(col)) + 0.1).astype(np.float32)
    return rowptr, col.astype(np.int32), val


def run_case(ctx, m, k, d, seed, long_rows, dtype):
    rowptr, col, val = block(m, k, seed, long_rows)
    t = lambda a: torch.as_tensor(a).to(DEV).contiguous()
    csr = plx.plx_csr_import(ctx, m, k, t(rowptr), t(col), t(val))
    assert plx.plx_csr_bins(csr, False)[0][1] + plx.plx_csr_bins(csr, False)[0][2] >= long_rows
    row = np.repeat(np.arange(m), np.diff(rowptr)); c64 = col.astype(np.int64); v64 = val.astype(np.float64)
    r = np.random.default_rng(seed + 1)
    X = torch.as_tensor(r.standard_normal((k, d)).astype(np.float32)).to(DEV).to(dtype)
    G = torch.as_tensor(r.standard_normal((m, d)).astype(np.float32)).to(DEV).to(dtype)
    Y = torch.empty(m, d, device=DEV, dtype=dtype); Yt = torch.empty(k, d, device=DEV, dtype=dtype)
    Ys = torch.full((m, d), 7.0, device=DEV, dtype=dtype); Yts = torch.full((k, d), 7.0, device=DEV, dtype=dtype)
    plx.plx_spmm(ctx, csr, X, Y); plx.plx_spmm_t(ctx, csr, G, Yt)
    plx.plx_sync(ctx)
    live, allocated = len(ctx._live), torch.cuda.memory_allocated()
    plx.plx_spmm_static(ctx, csr, False, X, Ys)
    plx.plx_spmm_static(ctx, csr, True, G, Yts)
    assert len(ctx._live) == live and torch.cuda.memory_allocated() == allocated      # nothing obtained from the allocator
    plx.plx_sync(ctx)
    # the bar of the existing entry points: same kernels, same order of additions => bit-identical
    assert torch.equal(Ys, Y) and torch.equal(Yts, Yt)
    tol = 1e-4 if dtype == torch.float32 else 2e-2
    ref = oracle.spmm_coo(m, row, c64, v64, X.float().cpu().numpy())
    ref_t = oracle.spmm_t_coo(k, row, c64, v64, G.float().cpu().numpy())
    assert rel_err(Ys, ref) <= tol and rel_err(Yts, ref_t) <= tol
    if dtype == torch.float32:
        assert elt_err(Ys, ref) <= 1e-3 and elt_err(Yts, ref_t) <= 1e-3
    csr.close()


def test_static_buffer_two_calls_second_smaller():
    ctx = plx.plx_ctx(0)
    run_case(ctx, 3000, 20000, 64, 5, 400, torch.float32)
    run_case(ctx, 700, 5000, 32, 6, 40, torch.float32)        # smaller, right after: stale partial sums would show
    run_case(ctx, 900, 6000, 100, 7, 60, torch.bfloat16)
    ctx.close()


def test_static_buffer_limit_is_an_error_before_any_work():
    """More segments than 32 MiB of partial sums hold: PLX_ERR_UNSUPPORTED, output untouched; the same handle at a
    narrower width fits and runs."""
    ctx = plx.plx_ctx(0)
    m, k = 9000, 8192
    r = np.random.default_rng(3)
    lens = np.full(m, 2100, np.int64)                          # every row: 8 windows, > 8 segments
    rowptr = np.zeros(m + 1, np.int64); rowptr[1:] = np.cumsum(lens)
    col = np.concatenate([np.sort(r.choice(k, 2100, replace=False)) for _ in range(m)]).astype(np.int32)
    val = (r.random(len(col)) + 0.1).astype(np.float32)
    t = lambda a: torch.as_tensor(a).to(DEV).contiguous()
    csr = plx.plx_csr_import(ctx, m, k, t(rowptr), t(col), t(val))
    X = torch.randn(k, 256, device=DEV)
    Y = torch.full((m, 256), 7.0, device=DEV)
    with pytest.raises(plx.PlxError) as err:                   # >= 72000 segments x 512 B (128 floats per pass) > 32 MiB
        plx.plx_spmm_static(ctx, csr, False, X, Y)
    assert err.value.status == plx.PLX_ERR_UNSUPPORTED and "fixed buffer" in str(err.value)
    plx.plx_sync(ctx)
    assert bool((Y == 7.0).all())
    Yn = torch.empty(m, 16, device=DEV); Yr = torch.empty(m, 16, device=DEV)
    plx.plx_spmm_static(ctx, csr, False, X[:, :16], Yn)        # 64 B per segment: fits
    plx.plx_spmm(ctx, csr, X[:, :16], Yr)
    plx.plx_sync(ctx)
    assert torch.equal(Yn, Yr)
    csr.close(); ctx.close()


def test_static_buffer_call_recorded_into_a_hip_graph():
    """What the entry point is for: a caller under HIP graph capture.  Both orientations of a block with split rows are
    recorded (nothing is allocated while recording), the graph is replayed with eager work and synchronisations in
    between, and every replay equals the eager plx_spmm / plx_spmm_t results bit for bit."""
    side = torch.cuda.Stream(device=DEV)
    ctx = plx.plx_ctx(0, stream=side.cuda_stream)
    m, k, d = 2000, 9000, 48
    rowptr, col, val = block(m, k, 21, 150)
    t = lambda a: torch.as_tensor(a).to(DEV).contiguous()
    csr = plx.plx_csr_import(ctx, m, k, t(rowptr), t(col), t(val))
    X = torch.randn(k, d, device=DEV); G = torch.randn(m, d, device=DEV)
    Y = torch.empty(m, d, device=DEV); Yt = torch.empty(k, d, device=DEV)
    Ys = torch.empty(m, d, device=DEV); Yts = torch.empty(k, d, device=DEV)
    torch.cuda.synchronize()
    plx.plx_spmm(ctx, csr, X, Y); plx.plx_spmm_t(ctx, csr, G, Yt); plx.plx_sync(ctx)
    live = len(ctx._live)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side, capture_error_mode="thread_local"):
        plx.plx_spmm_static(ctx, csr, False, X, Ys)
        plx.plx_spmm_static(ctx, csr, True, G, Yts)
    assert len(ctx._live) == live        # the library obtained nothing (torch's own graph bookkeeping allocates a little)
    for rep in range(3):
        Ys.fill_(float("nan")); Yts.fill_(float("nan"))                 # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Ys, Y) and torch.equal(Yts, Yt), f"replay {rep}"
    del graph
    csr.close(); ctx.close()
