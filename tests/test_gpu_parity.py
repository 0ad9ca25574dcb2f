"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Bit-exact for structure (row pointers, columns, degrees, fp32 values);
max|g-o| / max|o| <= 1e-4 for fp32 tensors (the tolerance the benchmark spec fixes)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import gcn as ogcn
import paper_2505_04083_amd as plx
import synth
from gcn_driver import elt_err, rel_err, run_network

pytestmark = pytest.mark.gpu
TOL32 = 1e-4
ELT32 = 1e-3        # element-wise form of the fp32 tolerance: |g - o| / max(|o|, 1e-3 max|o|)
BAND32 = 1e-5       # fp32: gradient entries whose |Q| is within this of zero (relative to max|Q|) are zeroed on both sides
DEV = "cuda:0"


def close(gpu, ref, tol):
    """The tolerance in both its forms: max-norm relative error <= tol, and for fp32 also the element-wise error
    |g - o| / max(|o|, 1e-3 max|o|) <= 1e-3 (an error in a small entry is weighed by that entry's own size)."""
    e = rel_err(gpu, ref)
    assert e <= tol, f"max-norm relative error {e:.3e} above {tol:g}"
    if tol == TOL32:
        e = elt_err(gpu, ref)
        assert e <= ELT32, f"element-wise relative error {e:.3e} above {ELT32:g}"


def band(dtype):
    """Width of the band around Q = 0 in which the two sides may take the integer decision of Eq. 2.4 differently:
    fp32 accumulation differs by ~1e-7 of the scale, a bf16-stored activation by ~4e-3."""
    return BAND32 if dtype == "f32" else 2e-2


@pytest.fixture(scope="module")
def ctx():
    c = plx.plx_ctx(0)
    yield c
    c.close()


def dev(a, dtype=None):
    t = torch.as_tensor(a)
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV).contiguous()


def bits(t):
    return t.cpu().numpy().view(np.uint32)


def noisy_edges(src, dst, seed=1):
    """Add reversed copies, duplicates and self-loops: the builder must drop them all."""
    r = np.random.default_rng(seed)
    k = max(1, len(src) // 10)
    pick = r.integers(0, len(src), k)
    loops = r.integers(0, max(int(src.max()), 1), k)
    s = np.concatenate([src, dst[pick], src[pick], loops])
    d = np.concatenate([dst, src[pick], dst[pick], loops])
    order = r.permutation(len(s))
    return s[order], d[order]


def graph_cases():
    tiny = synth.CONFIGS["tiny"]
    return {
        "tiny": tiny,
        "social_small": synth.CONFIGS["social"].scaled(0.05),       # hubs > 4096 entries: split rows
        "road_small": synth.CONFIGS["road"].scaled(2e-3),           # rows of 1..6 entries
    }


@pytest.mark.parametrize("name", ["tiny", "social_small", "road_small"])
def test_build_csr_bit_exact(ctx, name):
    cfg = graph_cases()[name]
    src, dst = (t.numpy() for t in cfg.edges())
    src, dst = noisy_edges(src, dst)
    pr, pc = (p.numpy() for p in cfg.perms())
    adj = oracle.adjacency(cfg.n, src, dst)
    csr = plx.plx_build_csr(ctx, cfg.n, dev(src), dev(dst), dev(pr), dev(pc))
    assert (csr.m, csr.k, csr.nnz) == (cfg.n, cfg.n, adj.nnz)
    for transposed, (a, b) in enumerate([(pr, pc), (pc, pr)]):
        rowptr, col, val = oracle.permuted_csr(adj, a, b)
        g_rowptr, g_col, g_val, g_deg = plx.plx_csr_export(ctx, csr, bool(transposed), with_deg=True)
        assert np.array_equal(g_rowptr.cpu().numpy(), rowptr)
        assert np.array_equal(g_col.cpu().numpy(), col)
        assert np.array_equal(bits(g_val), val.view(np.uint32))
        assert np.array_equal(g_deg.cpu().numpy(), adj.deg)
    # identity permutations (NULL)
    csr0 = plx.plx_build_csr(ctx, cfg.n, dev(src), dev(dst))
    rowptr, col, val = oracle.permuted_csr(adj)
    g = plx.plx_csr_export(ctx, csr0)
    assert np.array_equal(g[0].cpu().numpy(), rowptr) and np.array_equal(g[1].cpu().numpy(), col)
    assert np.array_equal(bits(g[2]), val.view(np.uint32))


def test_build_csr_degenerate_and_errors(ctx):
    e = torch.zeros(0, dtype=torch.int64, device=DEV)
    csr = plx.plx_build_csr(ctx, 5, e, e)                       # empty graph: A^ = I
    rowptr, col, val = plx.plx_csr_export(ctx, csr)
    assert rowptr.tolist() == [0, 1, 2, 3, 4, 5] and col.tolist() == [0, 1, 2, 3, 4] and val.tolist() == [1.0] * 5
    csr = plx.plx_build_csr(ctx, 0, e, e)
    assert (csr.m, csr.nnz) == (0, 0)
    loops = dev(np.array([1, 2, 2]))
    csr = plx.plx_build_csr(ctx, 3, loops, loops)               # only self-loops in the input
    assert csr.nnz == 3
    with pytest.raises(plx.PlxError) as err:
        plx.plx_build_csr(ctx, 3, dev(np.array([0, 3])), dev(np.array([1, 1])))
    assert err.value.status == plx.PLX_ERR_INVALID
    with pytest.raises(plx.PlxError) as err:
        plx.plx_build_csr(ctx, 3, dev(np.array([0])), dev(np.array([1])), dev(np.array([0, 0, 2])), None)
    assert err.value.status == plx.PLX_ERR_INVALID
    with pytest.raises(plx.PlxError) as err:
        plx.plx_build_csr(ctx, 3, dev(np.array([0])), dev(np.array([1])), None, dev(np.array([0, 1, 5])))
    assert err.value.status == plx.PLX_ERR_INVALID


def random_block(m, k, seed, empty_rows=True, giant_row=None):
    """Rectangular CSR block with skewed row lengths, some empty rows and optionally one very
    long row (more than the split threshold)."""
    r = np.random.default_rng(seed)
    lens = np.minimum(r.zipf(1.6, m), k // 2).astype(np.int64)
    if empty_rows:
        lens[r.integers(0, m, m // 7)] = 0
        lens[0] = 0; lens[m - 1] = 0
    if giant_row is not None:
        lens[giant_row] = min(k, 9000)
    rowptr = np.zeros(m + 1, np.int64); rowptr[1:] = np.cumsum(lens)
    col = np.concatenate([np.sort(r.choice(k, l, replace=False)) for l in lens if l > 0] or [np.zeros(0, np.int64)])
    val = r.random(len(col)).astype(np.float32) + 0.1
    return rowptr, col.astype(np.int32), val


def coo_of(rowptr, col, val):
    row = np.repeat(np.arange(len(rowptr) - 1), np.diff(rowptr))
    return row, col.astype(np.int64), val.astype(np.float64)


def test_import_transpose_bit_exact(ctx):
    m, k = 700, 12000
    rowptr, col, val = random_block(m, k, 3, giant_row=5)
    csr = plx.plx_csr_import(ctx, m, k, dev(rowptr), dev(col), dev(val))
    g = plx.plx_csr_export(ctx, csr, False)
    assert np.array_equal(g[0].cpu().numpy(), rowptr) and np.array_equal(g[1].cpu().numpy(), col)
    row, c64, _ = coo_of(rowptr, col, val)
    order = np.lexsort((row, c64))                     # transposed: sort by (col, row)
    t_rowptr = np.zeros(k + 1, np.int64); t_rowptr[1:] = np.cumsum(np.bincount(c64, minlength=k))
    gt = plx.plx_csr_export(ctx, csr, True)
    assert np.array_equal(gt[0].cpu().numpy(), t_rowptr)
    assert np.array_equal(gt[1].cpu().numpy(), row[order].astype(np.int32))
    assert np.array_equal(bits(gt[2]), val[order].view(np.uint32))
    (sub, wave, split), ent = plx.plx_csr_bins(csr, False)
    assert sub + wave + split == m and split >= 1 and wave >= 1 and sum(ent) == len(col)
    # structure errors are reported, not executed
    bad = col.copy(); bad[1], bad[2] = bad[2], bad[1]
    bad_rp = rowptr.copy(); bad_rp[3] = bad_rp[4] + 1
    for args in [(dev(rowptr), dev(bad), dev(val)), (dev(bad_rp), dev(col), dev(val))]:
        with pytest.raises(plx.PlxError) as err:
            plx.plx_csr_import(ctx, m, k, *args)
        assert err.value.status == plx.PLX_ERR_INVALID


def test_timing_trace_lists_launches_in_order(ctx):
    """plx_timing_trace: one line per timed launch, in launch order; the aggregated report of the same calls has the
    same names and counts; a buffer too small for all lines is an error, and either call clears the record."""
    import ctypes
    n = 3000
    src, dst = synth.rmat_edges(3, n, 20000)
    csr = plx.plx_build_csr(ctx, n, dev(src), dev(dst))
    X = torch.randn(n, 16, device=DEV); Y = torch.empty(n, 16, device=DEV)
    A = torch.randn(n, 40, device=DEV); B = torch.randn(40, 24, device=DEV); C = torch.empty(n, 24, device=DEV)
    def calls():
        plx.plx_spmm(ctx, csr, X, Y)
        plx.plx_gemm_nn(ctx, A, B, C)
        plx.plx_spmm_t(ctx, csr, X, Y)
    plx.plx_sync(ctx); plx.plx_timing_enable(ctx, True); plx.plx_timing_report(ctx)
    calls()
    trace = plx.plx_timing_trace(ctx)
    names = [name for name, _ in trace]
    g = [i for i, name in enumerate(names) if name.startswith("gemm_nn")]
    assert len(g) == 1 and 0 < g[0] < len(names) - 1                       # the dense product between the two sparse ones
    assert all(name.startswith("spmm_") and name.endswith("[A]") for name in names[:g[0]])
    assert all(name.startswith("spmm_") and name.endswith("[At]") for name in names[g[0] + 1:])
    assert all(ms > 0 for _, ms in trace)
    assert plx.plx_timing_trace(ctx) == []                                  # cleared
    calls()
    report = plx.plx_timing_report(ctx)
    assert {name: names.count(name) for name in names} == {name: cnt for name, (cnt, _) in report.items()}
    calls()
    small = ctypes.create_string_buffer(8)
    assert plx._lib.plx_timing_trace(ctx.handle, small, len(small)) == plx.PLX_ERR_SHAPE
    plx.plx_timing_report(ctx); plx.plx_timing_enable(ctx, False)
    csr.close()


@pytest.mark.parametrize("d,pad", [(1, 0), (2, 0), (4, 0), (8, 0), (8, 1), (16, 0), (32, 0), (41, 0), (41, 3), (47, 1), (64, 0), (100, 0),
                                   (128, 0), (128, 4), (300, 0), (30, 2)])
def test_spmm_and_transpose_parity(ctx, d, pad):
    """Width sweep over aligned, padded and unaligned layouts; block with empty rows, skewed
    rows and one split row; several tiles and a ragged tail."""
    m, k = 1531, 9973
    rowptr, col, val = random_block(m, k, 11 + d, giant_row=77)
    csr = plx.plx_csr_import(ctx, m, k, dev(rowptr), dev(col), dev(val))
    row, c64, v64 = coo_of(rowptr, col, val)
    r = np.random.default_rng(d)
    X = r.standard_normal((k, d)).astype(np.float32)
    G = r.standard_normal((m, d)).astype(np.float32)
    ld = d + pad
    Xd = torch.full((k, ld), float("nan"), device=DEV); Xd[:, :d] = dev(X)
    Gd = torch.full((m, ld), float("nan"), device=DEV); Gd[:, :d] = dev(G)
    Y = torch.full((m, ld), 7.0, device=DEV)
    Yt = torch.full((k, ld), 7.0, device=DEV)
    plx.plx_spmm(ctx, csr, Xd[:, :d], Y[:, :d])
    plx.plx_spmm_t(ctx, csr, Gd[:, :d], Yt[:, :d])
    plx.plx_sync(ctx)
    ref = oracle.spmm_coo(m, row, c64, v64, X)
    ref_t = oracle.spmm_t_coo(k, row, c64, v64, G)
    close(Y[:, :d], ref, TOL32)
    close(Yt[:, :d], ref_t, TOL32)
    if pad:
        assert bool((Y[:, d:] == 7.0).all()) and bool((Yt[:, d:] == 7.0).all())      # padding untouched
    assert bool((Y[0, :d] == 0).all())                                              # empty row -> zeros
    # run-to-run bit reproducibility (no floating-point atomics)
    Y2 = torch.empty_like(Y)
    plx.plx_spmm(ctx, csr, Xd[:, :d], Y2[:, :d]); plx.plx_sync(ctx)
    assert torch.equal(Y2[:, :d], Y[:, :d])


@pytest.mark.parametrize("n_blocks", [1, 3, 8, 64])
def test_blocked_aggregation(ctx, n_blocks):
    """Row-blocked aggregation (Sec. 5.2): each block's product against the oracle restricted to
    that block's rows; untouched rows stay untouched; all blocks together reproduce the
    unblocked result bit for bit; the stored structure is unchanged by re-blocking."""
    m, k, d = 1531, 9973, 48
    rowptr, col, val = random_block(m, k, 91, giant_row=1200)
    csr = plx.plx_csr_import(ctx, m, k, dev(rowptr), dev(col), dev(val))
    row, c64, v64 = coo_of(rowptr, col, val)
    r = np.random.default_rng(5)
    X = r.standard_normal((k, d)).astype(np.float32)
    G = r.standard_normal((m, d)).astype(np.float32)
    whole = torch.empty(m, d, device=DEV); whole_t = torch.empty(k, d, device=DEV)
    plx.plx_spmm(ctx, csr, dev(X), whole)
    plx.plx_spmm_t(ctx, csr, dev(G), whole_t)
    bins_before = plx.plx_csr_bins(csr, False), plx.plx_csr_bins(csr, True)
    plx.plx_csr_set_row_blocks(ctx, csr, n_blocks)
    assert (plx.plx_csr_bins(csr, False), plx.plx_csr_bins(csr, True)) == bins_before
    for t in (False, True):
        g = plx.plx_csr_export(ctx, csr, t)
        if not t:
            assert np.array_equal(g[0].cpu().numpy(), rowptr) and np.array_equal(g[1].cpu().numpy(), col)
            assert np.array_equal(bits(g[2]), val.view(np.uint32))
    ref = oracle.spmm_coo(m, row, c64, v64, X)
    ref_t = oracle.spmm_t_coo(k, row, c64, v64, G)
    for t, rows, src, full, want in ((False, m, X, whole, ref), (True, k, G, whole_t, ref_t)):
        nb, rpb = plx.plx_csr_row_blocks(csr, t)
        assert nb == n_blocks and rpb == -(-rows // n_blocks)
        Y = torch.full((rows, d), 7.0, device=DEV)
        for b in reversed(range(nb)):                               # any order
            lo, hi = min(rows, b * rpb), min(rows, (b + 1) * rpb)
            before = Y.clone()
            plx.plx_spmm_block(ctx, csr, t, b, dev(src), Y)
            plx.plx_sync(ctx)
            if hi > lo:
                close(Y[lo:hi], want[lo:hi], TOL32) or float(np.abs(want[lo:hi]).max()) == 0.0
            assert torch.equal(Y[:lo], before[:lo]) and torch.equal(Y[hi:], before[hi:])
        assert torch.equal(Y, full)
        # the whole-matrix entry points walk over the blocks
        Y2 = torch.empty_like(Y)
        (plx.plx_spmm_t if t else plx.plx_spmm)(ctx, csr, dev(src), Y2)
        plx.plx_sync(ctx)
        assert torch.equal(Y2, full)
    with pytest.raises(plx.PlxError) as err:
        plx.plx_spmm_block(ctx, csr, False, n_blocks, dev(X), whole)
    assert err.value.status == plx.PLX_ERR_INVALID
    with pytest.raises(plx.PlxError):
        plx.plx_csr_set_row_blocks(ctx, csr, 65)
    plx.plx_csr_set_row_blocks(ctx, csr, 1)
    Y3 = torch.empty_like(whole)
    plx.plx_spmm(ctx, csr, dev(X), Y3); plx.plx_sync(ctx)
    assert torch.equal(Y3, whole)
    csr.close()


@pytest.mark.parametrize("n_windows,n_blocks", [(1, 1), (2, 1), (3, 4), (8, 1), (13, 2), (64, 1)])
def test_column_windows(n_windows, n_blocks):
    """Rows of 256+ entries cut at column-window boundaries (and row blocks on top): every setting
    gives the oracle's product within the tolerance, reproducibly, and leaves the stored structure
    alone.  Many medium and a few very long rows, so each window holds segments of many rows."""
    m, k, d = 900, 30000, 40
    r = np.random.default_rng(n_windows)
    lens = np.minimum(r.zipf(1.3, m) * 40, k // 3).astype(np.int64)
    lens[5] = 17000; lens[6] = 0; lens[m - 1] = 5000
    rowptr = np.zeros(m + 1, np.int64); rowptr[1:] = np.cumsum(lens)
    col = np.concatenate([np.sort(r.choice(k, l, replace=False)) for l in lens if l > 0]).astype(np.int32)
    val = (r.random(len(col)) + 0.1).astype(np.float32)
    wctx = plx.plx_ctx(0)
    plx.plx_ctx_set_column_windows(wctx, n_windows)
    csr = plx.plx_csr_import(wctx, m, k, dev(rowptr), dev(col), dev(val))
    if n_blocks > 1:
        plx.plx_csr_set_row_blocks(wctx, csr, n_blocks)
    (sub, wave, split), ent = plx.plx_csr_bins(csr, False)
    assert wave >= 100 and split >= 2 and sum(ent) == len(col)
    row, c64, v64 = coo_of(rowptr, col, val)
    X = r.standard_normal((k, d)).astype(np.float32)
    G = r.standard_normal((m, d)).astype(np.float32)
    Y = torch.empty(m, d, device=DEV); Yt = torch.empty(k, d, device=DEV)
    plx.plx_spmm(wctx, csr, dev(X), Y)
    plx.plx_spmm_t(wctx, csr, dev(G), Yt)
    plx.plx_sync(wctx)
    close(Y, oracle.spmm_coo(m, row, c64, v64, X), TOL32)
    close(Yt, oracle.spmm_t_coo(k, row, c64, v64, G), TOL32)
    Y2 = torch.empty_like(Y); Yt2 = torch.empty_like(Yt)
    plx.plx_spmm(wctx, csr, dev(X), Y2); plx.plx_spmm_t(wctx, csr, dev(G), Yt2); plx.plx_sync(wctx)
    assert torch.equal(Y, Y2) and torch.equal(Yt, Yt2)
    g = plx.plx_csr_export(wctx, csr, False)
    assert np.array_equal(g[0].cpu().numpy(), rowptr) and np.array_equal(g[1].cpu().numpy(), col)
    with pytest.raises(plx.PlxError):
        plx.plx_ctx_set_column_windows(wctx, 65)
    csr.close(); wctx.close()


def test_spmm_eigenvector_pin(ctx):
    """A^ sqrt(d) = sqrt(d): the normalised adjacency built on the GPU, applied on the GPU."""
    cfg = synth.CONFIGS["tiny"]
    src, dst = cfg.edges(DEV)
    csr = plx.plx_build_csr(ctx, cfg.n, src, dst)
    deg = plx.plx_csr_export(ctx, csr, with_deg=True)[3]
    s = torch.sqrt(deg.double()).float().reshape(-1, 1).contiguous()
    y = torch.empty_like(s)
    plx.plx_spmm(ctx, csr, s, y); plx.plx_sync(ctx)
    assert float(((y - s).abs() / s).max()) < 5e-6


@pytest.mark.parametrize("M,N,K", [(1000, 128, 32), (517, 41, 128), (300, 128, 602), (129, 16, 128), (64, 47, 100),
                                   (2049, 32, 128), (5, 3, 7)])
def test_gemm_parity(ctx, M, N, K):
    r = np.random.default_rng(M + N + K)
    A = r.standard_normal((M, K)).astype(np.float32)
    B = r.standard_normal((K, N)).astype(np.float32)
    C = torch.empty(M, N, device=DEV)
    plx.plx_gemm_nn(ctx, dev(A), dev(B), C)
    close(C, oracle.gemm(A, B), TOL32)
    Bt = np.ascontiguousarray(B.T)
    C2 = torch.empty(M, N, device=DEV)
    plx.plx_gemm_nt(ctx, dev(A), dev(Bt), C2)
    close(C2, oracle.gemm(A, Bt, tb=True), TOL32)
    # transposed product: reduction over the M rows
    G = r.standard_normal((M, N)).astype(np.float32)
    dW = torch.empty(K, N, device=DEV)
    plx.plx_gemm_tn(ctx, dev(A), dev(G), dW)
    close(dW, oracle.gemm(A, G, ta=True), TOL32)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,N,K", [(300, 128, 602), (1000, 200, 70), (513, 130, 300), (64, 129, 133), (129, 33, 37),
                                   (257, 602, 128), (128, 64, 256), (385, 96, 32), (1, 1, 1), (131, 100, 601)])
def test_gemm_deep_products_on_aligned_padded_rows(ctx, M, N, K, dtype):
    """The products outside the layer-sized range (K or N above 128, and every A B^T) on 16-byte
    aligned rows take the slab kernel with 128-bit buffer loads; with bf16 storage the inputs are
    widened on load and the results rounded to bf16.  Rows are padded to a multiple of 16 bytes
    (plus one more piece for odd sizes) and the padding holds NaN: a piece that straddles K, a row
    past M or a column past N that reached a product, or a store outside the result's width, shows
    up.  The oracle sees the stored (bf16-rounded) inputs in fp64."""
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    tol = TOL32 if dtype == "f32" else 2e-2
    r = np.random.default_rng(3 * M + 5 * N + 7 * K)

    def padded(a, t=tdt):
        q = 4 if t == torch.float32 else 8
        ld = -(-a.shape[1] // q) * q + q * ((M + N + K) % 2)
        buf = torch.full((a.shape[0], ld), float("nan"), dtype=t, device=DEV)
        buf[:, :a.shape[1]] = torch.as_tensor(a.astype(np.float32)).to(t).to(DEV)
        return buf, buf[:, :a.shape[1]]

    B = r.standard_normal((K, N)).astype(np.float32)          # the weight operand is fp32 in both modes
    (_, Av), (_, Gv) = padded(r.standard_normal((M, K))), padded(r.standard_normal((M, N)))
    (_, Bv), (_, Btv) = padded(B, torch.float32), padded(np.ascontiguousarray(B.T), torch.float32)
    A64, G64 = Av.double().cpu().numpy(), Gv.double().cpu().numpy()
    Cp, Cv = padded(np.zeros((M, N)))
    plx.plx_gemm_nn(ctx, Av, Bv, Cv)
    close(Cv.float(), oracle.gemm(A64, B), tol)
    assert bool(torch.isnan(Cp[:, N:].float()).all())
    Cp2, Cv2 = padded(np.zeros((M, N)))
    plx.plx_gemm_nt(ctx, Av, Btv, Cv2)
    close(Cv2.float(), oracle.gemm(A64, np.ascontiguousarray(B.T), tb=True), tol)
    assert bool(torch.isnan(Cp2[:, N:].float()).all())
    dWp, dWv = padded(np.zeros((K, N)), torch.float32)
    plx.plx_gemm_tn(ctx, Av, Gv, dWv)
    close(dWv, oracle.gemm(A64, G64, ta=True), tol)
    assert bool(torch.isnan(dWp[:, N:]).all())


def test_gemm_bf16_wide_products_need_aligned_rows(ctx):
    """bf16 products beyond the layer-sized kernels exist only for 16-byte aligned rows: anything else
    is refused with PLX_ERR_UNSUPPORTED, nothing is computed on a slower path."""
    A = torch.zeros(64, 301, dtype=torch.bfloat16, device=DEV)        # 602-byte rows
    B = torch.zeros(301, 128, device=DEV)
    C = torch.zeros(64, 128, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(plx.PlxError) as e:
        plx.plx_gemm_nn(ctx, A, B, C)
    assert e.value.status == plx.PLX_ERR_UNSUPPORTED
    with pytest.raises(plx.PlxError) as e:
        plx.plx_gemm_tn(ctx, A, C, torch.zeros(301, 128, device=DEV))
    assert e.value.status == plx.PLX_ERR_UNSUPPORTED


def test_gemm_tn_long_reduction_and_padding(ctx):
    R, M, N = 300_000, 32, 128
    A = synth.normal(5, 1, R, M, DEV)
    Bfull = torch.zeros(R, N + 4, device=DEV)
    Bfull[:, :N] = synth.normal(5, 2, R, N, DEV)
    C = torch.empty(M, N, device=DEV)
    plx.plx_gemm_tn(ctx, A, Bfull[:, :N], C)
    ref = oracle.gemm(A.cpu().numpy(), Bfull[:, :N].cpu().numpy(), ta=True)
    close(C, ref, TOL32)
    C2 = torch.empty_like(C)
    plx.plx_gemm_tn(ctx, A, Bfull[:, :N], C2)
    assert torch.equal(C, C2)


def test_elementwise_parity(ctx):
    r = np.random.default_rng(0)
    Z = r.standard_normal((1001, 47)).astype(np.float32); Z[3, 4] = 0.0
    dF = r.standard_normal((1001, 47)).astype(np.float32)
    F = torch.empty(1001, 47, device=DEV); dZ = torch.empty(1001, 47, device=DEV)
    plx.plx_relu(ctx, dev(Z), F); plx.plx_relu_bwd(ctx, dev(Z), dev(dF), dZ)
    assert np.array_equal(F.cpu().numpy(), oracle.relu(Z).astype(np.float32))
    assert np.array_equal(dZ.cpu().numpy(), oracle.relu_bwd(Z, dF).astype(np.float32))
    # padded layout takes the 2-D kernel
    Zp = torch.zeros(1001, 50, device=DEV); Zp[:, :47] = dev(Z)
    Fp = torch.full((1001, 50), 9.0, device=DEV)
    plx.plx_relu(ctx, Zp[:, :47], Fp[:, :47])
    assert torch.equal(Fp[:, :47], F) and bool((Fp[:, 47:] == 9.0).all())
    y = r.integers(0, 47, 1001)
    g = torch.empty(1001, 47, device=DEV); loss = torch.zeros(1, device=DEV)
    plx.plx_softmax_ce(ctx, dev(Z * 3), dev(y), g, loss=loss); plx.plx_sync(ctx)
    ref_loss, ref_g = oracle.softmax_ce(Z.astype(np.float64) * 3, y)
    close(g, ref_g, TOL32)
    assert abs(loss.item() - ref_loss) / ref_loss <= TOL32


@pytest.mark.parametrize("c", [1, 5, 16, 41, 47, 128, 130, 257, 1000])
@pytest.mark.parametrize("padded", [False, True])
def test_softmax_ce_widths_and_layouts(ctx, c, padded):
    """Loss head (Sec. 2.1) over class counts on both sides of every lane-group size, in contiguous
    rows (the scalar kernel unless c is a multiple of 4) and in rows padded to 16 bytes (the 128-bit
    kernel up to 256 classes); the padding holds NaN on input and must stay untouched on output."""
    n = 1237
    r = np.random.default_rng(c)
    Z = (r.standard_normal((n, c)) * 4).astype(np.float32)
    y = r.integers(0, c, n)
    ld = -(-c // 4) * 4 + (4 if padded else 0) if padded else c
    Zd = torch.full((n, ld), float("nan"), device=DEV); Zd[:, :c] = dev(Z)
    g = torch.full((n, ld), 7.0, device=DEV)
    loss = torch.zeros(1, device=DEV)
    plx.plx_softmax_ce(ctx, Zd[:, :c], dev(y), g[:, :c], loss=loss); plx.plx_sync(ctx)
    ref_loss, ref_g = oracle.softmax_ce(Z.astype(np.float64), y)
    close(g[:, :c], ref_g, TOL32)
    assert abs(loss.item() - ref_loss) <= TOL32 * max(1.0, abs(ref_loss))
    assert bool((g[:, c:] == 7.0).all())


@pytest.mark.parametrize("c", [1, 5, 16, 41, 47, 128, 130, 257, 600])
@pytest.mark.parametrize("padded", [False, True])
def test_softmax_ce_bf16_widths_and_layouts(ctx, c, padded):
    """The loss head on bf16 logits: contiguous rows (the scalar kernel unless c is a multiple of 8) and rows padded to
    16 bytes (eight classes per lane, 128-bit accesses, up to 512 classes).  The oracle sees the logits as stored; the
    gradient comes back rounded to bf16 (2^-9 of an element), the loss in fp32; padding holds NaN on input and must stay
    untouched on output."""
    n = 1237
    r = np.random.default_rng(100 + c)
    Zb = torch.from_numpy((r.standard_normal((n, c)) * 4).astype(np.float32)).to(torch.bfloat16)
    y = r.integers(0, c, n)
    ld = -(-c // 8) * 8 + 8 if padded else c
    Zd = torch.full((n, ld), float("nan"), device=DEV, dtype=torch.bfloat16); Zd[:, :c] = Zb.to(DEV)
    g = torch.full((n, ld), 7.0, device=DEV, dtype=torch.bfloat16)
    loss = torch.zeros(1, device=DEV)
    plx.plx_softmax_ce(ctx, Zd[:, :c], dev(y), g[:, :c], loss=loss); plx.plx_sync(ctx)
    ref_loss, ref_g = oracle.softmax_ce(Zb.double().numpy(), y)
    assert rel_err(g[:, :c].float(), ref_g) <= 4e-3
    assert abs(loss.item() - ref_loss) <= TOL32 * max(1.0, abs(ref_loss))
    assert bool((g[:, c:] == 7.0).all())


@pytest.mark.parametrize("order", [plx.PLX_ORDER_COMBINE_FIRST, plx.PLX_ORDER_AGG_FIRST, plx.PLX_ORDER_AUTO])
def test_three_layer_network_parity(ctx, order):
    """configs[0]: R-MAT N=4096, 65,536 edges, 128-128-128-16, one forward + backward, against
    the oracle on the UNPERMUTED graph (Eq. 5.3-5.4 give the index maps)."""
    cfg = synth.CONFIGS["tiny"]
    src, dst = cfg.edges()
    pr, pc = cfg.perms()
    F0, Ws, y = cfg.features(), cfg.weights(), cfg.labels()
    adj = oracle.adjacency(cfg.n, src.numpy(), dst.numpy())
    assert adj.nnz == 135168
    ref = ogcn.forward_backward(adj, F0.numpy(), [w.numpy() for w in Ws], y.numpy())

    csr = plx.plx_build_csr(ctx, cfg.n, src.to(DEV), dst.to(DEV), pr.to(DEV), pc.to(DEV))
    H0 = torch.empty_like(F0); H0[pc] = F0                        # P_c F0
    L = len(Ws)
    out_perm = pr if (L - 1) % 2 == 0 else pc
    y_gpu = torch.empty_like(y); y_gpu[out_perm] = y
    run = run_network(ctx, csr, H0.to(DEV), [w.to(DEV) for w in Ws], y_gpu.to(DEV), order=order)
    for l in range(L):
        perm = (pr if l % 2 == 0 else pc).to(DEV)
        close(run.Z[l][perm], ref.Q[l], TOL32), f"Z of layer {l}"
    assert abs(run.loss.item() - ref.loss) / ref.loss <= TOL32
    for l in range(L):
        close(run.dW[l], ref.dW[l], TOL32), f"dW of layer {l}"
    close(run.dF0[pc.to(DEV)], ref.dF[0], TOL32)


def test_three_layer_network_as_the_bench_runs_it(ctx):
    """configs[0] through the sequencer's default storage (activations only, sign bits, and the
    backward chain that never forms the gradient between layers 1 and 2) against the oracle, and
    against the same network with the chain switched off."""
    from paper_2505_04083_amd.network import GcnNetwork
    cfg = synth.CONFIGS["tiny"]
    src, dst = cfg.edges()
    pr, pc = cfg.perms()
    F0, Ws, y = cfg.features(), cfg.weights(), cfg.labels()
    adj = oracle.adjacency(cfg.n, src.numpy(), dst.numpy())
    ref = ogcn.forward_backward(adj, F0.numpy(), [w.numpy() for w in Ws], y.numpy())
    csr = plx.plx_build_csr(ctx, cfg.n, src.to(DEV), dst.to(DEV), pr.to(DEV), pc.to(DEV))
    H0 = torch.empty_like(F0); H0[pc] = F0
    L = len(Ws)
    y_gpu = torch.empty_like(y); y_gpu[pr if (L - 1) % 2 == 0 else pc] = y
    nets = []
    for chain in (True, False):
        net = GcnNetwork(ctx, csr, [w.to(DEV) for w in Ws], chain=chain)
        net.step(H0.to(DEV), y_gpu.to(DEV)); net.sync()
        nets.append(net)
        assert abs(net.loss.item() - ref.loss) / ref.loss <= TOL32
        for l in range(L):
            close(net.dW[l], ref.dW[l], TOL32), f"dW of layer {l}, chain={chain}"
        close(net.dH[0][pc.to(DEV)], ref.dF[0], TOL32)
    assert nets[0].chained == [False, True, False] and nets[0].dH[2] is None and nets[0].dT[2] is not None
    assert nets[0].fwd_chained == [False, True, False] and nets[0].T[2] is not None
    assert nets[1].chained == [False, False, False] and nets[1].fwd_chained == [False, False, False]
    assert rel_err(nets[0].Z[-1], nets[1].Z[-1].double().cpu().numpy()) <= 2e-5
    for l in range(L):
        assert rel_err(nets[0].dW[l], nets[1].dW[l].double().cpu().numpy()) <= 2e-5


@pytest.mark.parametrize("dims", [(128, 128, 128, 16), (64, 128, 16), (200, 64, 10)])
def test_network_without_the_input_feature_gradient(ctx, dims):
    """GcnNetwork(input_grad=False) leaves out Eq. 2.6-2.7 of the first layer only: logits, loss and every dW are those of
    the full backward pass bit for bit (the same kernels form them), dW also agrees with the oracle, and dH[0] does not
    exist.  The shapes cover a first layer in aggregate-first order with and without the chained kernel behind it
    (64-128-16 is the road network's: its fused backward kernel then runs without its Eq. 2.6 product) and one in
    combine-first order (200 -> 64)."""
    from paper_2505_04083_amd.network import GcnNetwork
    n = 3000
    src, dst = synth.rmat_edges(11, n, 24000)
    g = torch.Generator().manual_seed(5)
    pr, pc = torch.randperm(n, generator=g), torch.randperm(n, generator=g)
    F0 = torch.randn(n, dims[0], generator=g)
    Ws = [torch.randn(dims[l], dims[l + 1], generator=g) / dims[l] ** 0.5 for l in range(len(dims) - 1)]
    y = torch.randint(0, dims[-1], (n,), generator=g)
    adj = oracle.adjacency(n, src.numpy(), dst.numpy())
    ref = ogcn.forward_backward(adj, F0.numpy(), [w.numpy() for w in Ws], y.numpy())
    csr = plx.plx_build_csr(ctx, n, dev(src), dev(dst), dev(pr), dev(pc))
    H0 = torch.empty_like(F0); H0[pc] = F0
    L = len(Ws)
    y_gpu = torch.empty_like(y); y_gpu[pr if (L - 1) % 2 == 0 else pc] = y
    full = GcnNetwork(ctx, csr, [dev(w) for w in Ws])
    lean = GcnNetwork(ctx, csr, [dev(w) for w in Ws], input_grad=False)
    for net in (full, lean):
        net.step(dev(H0), dev(y_gpu)); net.sync()
    assert lean.dH[0] is None and full.dH[0] is not None
    assert torch.equal(lean.Z[-1], full.Z[-1]) and lean.loss.item() == full.loss.item()
    for l in range(L):
        assert torch.equal(lean.dW[l], full.dW[l]), f"dW of layer {l}"
        close(lean.dW[l], ref.dW[l], TOL32)
    close(full.dH[0][dev(pc)], ref.dF[0], TOL32)
    csr.close()


def test_layer_on_rectangular_block_both_orders(ctx):
    """One layer on an imported rectangular block (the shape of configs[3], shrunk): forward
    and backward in both multiplication orders against the oracle's Eq. 2.1-2.7."""
    m, k, din, dout = 2100, 8300, 32, 128
    rowptr, col, val = random_block(m, k, 5, giant_row=9)
    csr = plx.plx_csr_import(ctx, m, k, dev(rowptr), dev(col), dev(val))
    row, c64, v64 = coo_of(rowptr, col, val)
    r = np.random.default_rng(1)
    X = r.standard_normal((k, din)).astype(np.float32)
    W = (r.standard_normal((din, dout)) * 0.2).astype(np.float32)
    dFn = r.standard_normal((m, dout)).astype(np.float32)
    Hagg = oracle.spmm_coo(m, row, c64, v64, X)
    Q = oracle.gemm(Hagg, W)
    dQ = oracle.relu_bwd(Q, dFn)
    dW = oracle.gemm(Hagg, dQ, ta=True)
    dX = oracle.spmm_t_coo(k, row, c64, v64, oracle.gemm(dQ, W, tb=True))
    for order in (plx.PLX_ORDER_AGG_FIRST, plx.PLX_ORDER_COMBINE_FIRST):
        ws = torch.empty(plx.plx_gcn_layer_workspace(csr, False, din, dout, order=order), dtype=torch.uint8, device=DEV)
        Z = torch.empty(m, dout, device=DEV); F = torch.empty(m, dout, device=DEV)
        saved = torch.empty(m, din, device=DEV)
        plx.plx_gcn_layer_fwd(ctx, csr, False, dev(X), dev(W), Z, F, saved, ws, order=order)
        gdX = torch.empty(k, din, device=DEV); gdW = torch.empty(din, dout, device=DEV)
        plx.plx_gcn_layer_bwd(ctx, csr, False, dev(X), dev(W), Z, dev(dFn), saved, gdX, gdW, ws, order=order)
        plx.plx_sync(ctx)
        close(Z, Q, TOL32)
        close(F, oracle.relu(Q), TOL32)
        close(gdW, dW, TOL32)
        close(gdX, dX, TOL32)
        # only the activated output stored; the backward call takes it in place of Z
        F2 = torch.empty(m, dout, device=DEV)
        plx.plx_gcn_layer_fwd(ctx, csr, False, dev(X), dev(W), None, F2, saved, ws, order=order)
        gdX2 = torch.empty(k, din, device=DEV); gdW2 = torch.empty(din, dout, device=DEV)
        plx.plx_gcn_layer_bwd(ctx, csr, False, dev(X), dev(W), F2, dev(dFn), saved, gdX2, gdW2, ws, order=order)
        plx.plx_sync(ctx)
        assert torch.equal(F2, F) and torch.equal(gdX2, gdX) and torch.equal(gdW2, gdW)
        # weight gradient only
        gdW3 = torch.empty(din, dout, device=DEV)
        plx.plx_gcn_layer_bwd(ctx, csr, False, dev(X), dev(W), F2, dev(dFn), saved, None, gdW3, ws, order=order)
        plx.plx_sync(ctx)
        assert torch.equal(gdW3, gdW)


@pytest.mark.parametrize("din,dout", [(32, 128), (128, 128), (100, 47), (128, 16), (64, 128), (33, 65), (602, 128)])
def test_layer_backward_shapes(ctx, din, dout):
    """Backward of one layer over the width pairs of the five workloads (ragged widths, widths
    above the fused kernel's range fall back to the separate products), both orders."""
    m, k = 1300, 1700
    rowptr, col, val = random_block(m, k, din + dout)
    csr = plx.plx_csr_import(ctx, m, k, dev(rowptr), dev(col), dev(val))
    row, c64, v64 = coo_of(rowptr, col, val)
    r = np.random.default_rng(din * 7 + dout)
    X = r.standard_normal((k, din)).astype(np.float32)
    W = (r.standard_normal((din, dout)) * 0.2).astype(np.float32)
    dFn = r.standard_normal((m, dout)).astype(np.float32)
    Hagg = oracle.spmm_coo(m, row, c64, v64, X)
    Q = oracle.gemm(Hagg, W)
    dQ = oracle.relu_bwd(Q, dFn)
    dW = oracle.gemm(Hagg, dQ, ta=True)
    dX = oracle.spmm_t_coo(k, row, c64, v64, oracle.gemm(dQ, W, tb=True))
    for order in (plx.PLX_ORDER_AGG_FIRST, plx.PLX_ORDER_COMBINE_FIRST):
        ws = torch.empty(plx.plx_gcn_layer_workspace(csr, False, din, dout, order=order), dtype=torch.uint8, device=DEV)
        F = torch.empty(m, dout, device=DEV); saved = torch.empty(m, din, device=DEV)
        plx.plx_gcn_layer_fwd(ctx, csr, False, dev(X), dev(W), None, F, saved, ws, order=order)
        gdX = torch.empty(k, din, device=DEV); gdW = torch.empty(din, dout, device=DEV)
        plx.plx_gcn_layer_bwd(ctx, csr, False, dev(X), dev(W), F, dev(dFn), saved, gdX, gdW, ws, order=order)
        plx.plx_sync(ctx)
        close(F, oracle.relu(Q), TOL32)
        close(gdW, dW, TOL32)
        close(gdX, dX, TOL32)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("din,dout", [(100, 47), (33, 65), (128, 41)])
def test_layer_ragged_widths_in_padded_rows(ctx, din, dout, dtype):
    """Ragged widths stored with a padded leading dimension (what the network sequencer does): the
    padding holds NaN, so any padding element that reaches a product or any result written outside
    its width shows up.  Covers the whole-chunk-then-mask loads and the single-element path of the
    matrix's last row."""
    m, k = 777, 1111
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    code = plx.PLX_F32 if dtype == "f32" else plx.PLX_BF16
    tol = TOL32 if dtype == "f32" else 2e-2
    rowptr, col, val = random_block(m, k, 5 * din + dout)
    csr = plx.plx_csr_import(ctx, m, k, dev(rowptr), dev(col), dev(val))
    row, c64, v64 = coo_of(rowptr, col, val)
    r = np.random.default_rng(din + 3 * dout)

    def padded(a, width):
        ld = -(-width // 16) * 16
        t = torch.full((a.shape[0], ld), float("nan"), dtype=tdt, device=DEV)
        t[:, :width] = torch.as_tensor(a.astype(np.float32)).to(tdt).to(DEV)
        return t, t[:, :width].double().cpu().numpy()

    Xp, X64 = padded(r.standard_normal((k, din)), din)
    W = (r.standard_normal((din, dout)) * 0.2).astype(np.float32)
    Hagg = oracle.spmm_coo(m, row, c64, v64, X64)
    Q = oracle.gemm(Hagg, W)
    dF = r.standard_normal((m, dout)) * (np.abs(Q) > band(dtype) * np.abs(Q).max())     # keep clear of the mask's rounding band
    dFp, dF64 = padded(dF, dout)
    dQ = oracle.relu_bwd(Q, dF64)
    dW = oracle.gemm(Hagg, dQ, ta=True)
    dX = oracle.spmm_t_coo(k, row, c64, v64, oracle.gemm(dQ, W, tb=True))
    for order in (plx.PLX_ORDER_AGG_FIRST, plx.PLX_ORDER_COMBINE_FIRST):
        ws = torch.empty(plx.plx_gcn_layer_workspace(csr, False, din, dout, dtype=code, order=order), dtype=torch.uint8, device=DEV)
        Fp, _ = padded(np.zeros((m, dout)), dout)
        Sp, _ = padded(np.zeros((m, din)), din)
        gXp, _ = padded(np.zeros((k, din)), din)
        gdW = torch.empty(din, dout, device=DEV)
        plx.plx_gcn_layer_fwd(ctx, csr, False, Xp[:, :din], dev(W), None, Fp[:, :dout], Sp[:, :din], ws, order=order)
        plx.plx_gcn_layer_bwd(ctx, csr, False, Xp[:, :din], dev(W), Fp[:, :dout], dFp[:, :dout], Sp[:, :din], gXp[:, :din],
                              gdW, ws, order=order)
        plx.plx_sync(ctx)
        close(Fp[:, :dout].float(), oracle.relu(Q), tol)
        close(gdW, dW, tol)
        close(gXp[:, :din].float(), dX, tol)
        for t, wdt in ((Fp, dout), (gXp, din)):                                 # padding untouched
            assert bool(torch.isnan(t[:, wdt:].float()).all())


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("din,dout", [(32, 128), (128, 128), (100, 47), (33, 65), (16, 16), (128, 16), (64, 96), (602, 128)])
def test_layer_sign_bits(ctx, din, dout, dtype):
    """ReLU kept as one sign bit per element: the words the forward call writes are exactly the packed
    [F > 0] of the activated output it writes beside them (zero beyond the width, nothing written
    beyond the words of a row), and the backward call fed with the words returns bit for bit what it
    returns when fed with the value matrix; results are checked against the oracle as well.  Widths
    cover both fused dense kernels, the general product (602: separate sign pass) and both orders."""
    m, k = 1237, 1500                                # several tiles and a ragged last one
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16

    def matrix(rows, cols, t=tdt):                   # bf16 widths above 128 need 16-byte aligned rows
        ld = -(-cols // 8) * 8 if (dtype == "bf16" and max(din, dout) > 128) else cols
        return torch.zeros(rows, ld, dtype=t, device=DEV)[:, :cols]

    code = plx.PLX_F32 if dtype == "f32" else plx.PLX_BF16
    tol = TOL32 if dtype == "f32" else 2e-2
    rowptr, col, val = random_block(m, k, 11 * din + dout)
    csr = plx.plx_csr_import(ctx, m, k, dev(rowptr), dev(col), dev(val))
    row, c64, v64 = coo_of(rowptr, col, val)
    r = np.random.default_rng(5 * din + dout)
    X = matrix(k, din); X.copy_(torch.as_tensor(r.standard_normal((k, din)).astype(np.float32)))
    X64 = X.double().cpu().numpy()
    W = (r.standard_normal((din, dout)) * 0.2).astype(np.float32)
    Hagg = oracle.spmm_coo(m, row, c64, v64, X64)
    Q = oracle.gemm(Hagg, W)
    dF64 = r.standard_normal((m, dout)) * (np.abs(Q) > band(dtype) * np.abs(Q).max())   # keep clear of the mask's rounding band
    dF = matrix(m, dout); dF.copy_(torch.as_tensor(dF64.astype(np.float32)))
    dF64 = dF.double().cpu().numpy()
    dQ = oracle.relu_bwd(Q, dF64)
    dW = oracle.gemm(Hagg, dQ, ta=True)
    dX = oracle.spmm_t_coo(k, row, c64, v64, oracle.gemm(dQ, W, tb=True))
    nw = (dout + 31) // 32
    for order in (plx.PLX_ORDER_AGG_FIRST, plx.PLX_ORDER_COMBINE_FIRST):
        ws = torch.empty(plx.plx_gcn_layer_workspace(csr, False, din, dout, dtype=code, act=plx.PLX_ACT_RELU_BITS, order=order),
                         dtype=torch.uint8, device=DEV)
        F = matrix(m, dout); saved = matrix(m, din)
        words = torch.full((m, nw + 1), 0x5A5A5A5A, dtype=torch.int32, device=DEV)
        plx.plx_gcn_layer_fwd(ctx, csr, False, X, dev(W), words[:, :nw], F, saved, ws, act=plx.PLX_ACT_RELU_BITS, order=order)
        outs = []
        for act, mask in ((plx.PLX_ACT_RELU_BITS, words[:, :nw]), (plx.PLX_ACT_RELU, F)):
            gdX = matrix(k, din); gdW = torch.empty(din, dout, device=DEV)
            plx.plx_gcn_layer_bwd(ctx, csr, False, X, dev(W), mask, dF, saved, gdX, gdW, ws, act=act, order=order)
            outs.append((gdX, gdW))
        plx.plx_sync(ctx)
        pos = (F.float() > 0).cpu().numpy()
        padded = np.zeros((m, 32 * nw), dtype=np.uint64)
        padded[:, :dout] = pos
        want = (padded.reshape(m, nw, 32) << np.arange(32, dtype=np.uint64)).sum(axis=2).astype(np.uint32)
        got = words.cpu().numpy().view(np.uint32)
        assert np.array_equal(got[:, :nw], want)
        assert np.all(got[:, nw] == 0x5A5A5A5A)
        close(F.float(), oracle.relu(Q), tol)
        assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
        close(outs[0][1], dW, tol)
        close(outs[0][0].float(), dX, tol)


@pytest.mark.parametrize("din,dout,dn,dtype,act", [
    (64, 128, 16, "f32", "bits"), (128, 128, 32, "f32", "bits"), (100, 128, 17, "f32", "bits"), (128, 128, 41, "f32", "bits"),
    (64, 96, 16, "f32", "bits"), (96, 128, 31, "f32", "none"), (64, 128, 3, "f32", "bits"),
    (32, 128, 16, "f32", "bits"), (64, 64, 16, "f32", "bits"), (128, 128, 100, "f32", "bits"), (64, 128, 16, "f32", "values"),
    (602, 128, 16, "f32", "bits"), (64, 128, 16, "bf16", "bits"), (64, 128, 16, "f32", "bits-combine")])
def test_chained_backward_of_two_layers(ctx, din, dout, dn, dtype, act):
    """Backward of two consecutive layers without the gradient between them: the second layer
    (combine-first, transposed adjacency) stops at dT = A^T dZ, the first takes (dT, Wn) in place of dF.
    Shapes cover the fused kernel (one and two 16-column steps of dn, ragged dn and widths, a
    wavefront without columns, no mask) and every fall-back (narrow widths, wide dn, value mask,
    general products, bf16, combine-first order).  Checked against the oracle and against the
    unchained calls."""
    m, k = 1237, 1500
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    code = plx.PLX_F32 if dtype == "f32" else plx.PLX_BF16
    tol = TOL32 if dtype == "f32" else 2e-2
    order = plx.PLX_ORDER_COMBINE_FIRST if act.endswith("combine") else plx.PLX_ORDER_AGG_FIRST
    actc = {"bits": plx.PLX_ACT_RELU_BITS, "bits-combine": plx.PLX_ACT_RELU_BITS, "values": plx.PLX_ACT_RELU, "none": plx.PLX_ACT_NONE}[act]
    rowptr, col, val = random_block(m, k, 3 * din + 5 * dout + dn)
    csr = plx.plx_csr_import(ctx, m, k, dev(rowptr), dev(col), dev(val))
    row, c64, v64 = coo_of(rowptr, col, val)
    r = np.random.default_rng(din + dout + dn)

    def matrix(rows, cols, src=None, t=tdt):         # rows padded to 16 bytes, as the network keeps them
        q = 16 // torch.empty(0, dtype=t).element_size()
        buf = torch.zeros(rows, -(-cols // q) * q, dtype=t, device=DEV)[:, :cols]
        if src is not None:
            buf.copy_(torch.as_tensor(np.asarray(src, np.float32)))
        return buf

    X = matrix(k, din, r.standard_normal((k, din)))
    W = (r.standard_normal((din, dout)) * 0.2).astype(np.float32)
    Wn = (r.standard_normal((dout, dn)) * 0.2).astype(np.float32)
    dZn = matrix(k, dn, r.standard_normal((k, dn)))
    X64, dZn64 = X.double().cpu().numpy(), dZn.double().cpu().numpy()
    # oracle: layer l (A, ReLU or none), layer l+1 (A^T, combine-first, no activation); F is taken from the GPU's
    # stored activation for the second layer's products, so that bf16 storage rounding is shared
    S = oracle.spmm_coo(m, row, c64, v64, X64)
    Q = oracle.gemm(S, W)
    nbytes = plx.plx_gcn_layer_bwd_chained_workspace(ctx, csr, False, din, dout, dn, dtype=code, act=actc, order=order)
    ws1 = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    ws2 = torch.empty(plx.plx_gcn_layer_workspace(csr, True, dout, dn, dtype=code, act=plx.PLX_ACT_NONE,
                                                  order=plx.PLX_ORDER_COMBINE_FIRST), dtype=torch.uint8, device=DEV)
    F = matrix(m, dout); saved = matrix(m, din)
    words = torch.zeros(m, (dout + 31) // 32, dtype=torch.int32, device=DEV)
    Zarg = words if actc == plx.PLX_ACT_RELU_BITS else None
    plx.plx_gcn_layer_fwd(ctx, csr, False, X, dev(W), Zarg, F, saved, ws1, act=actc, order=order)
    mask_src = {plx.PLX_ACT_RELU_BITS: words, plx.PLX_ACT_RELU: F, plx.PLX_ACT_NONE: None}[actc]
    # chained
    dT = matrix(m, dn); gdWn = torch.empty(dout, dn, device=DEV)
    plx.plx_gcn_layer_bwd_dt(ctx, csr, True, F, None, dZn, dT, gdWn, ws2, act=plx.PLX_ACT_NONE)
    gdX = matrix(k, din); gdW = torch.empty(din, dout, device=DEV)
    plx.plx_sync(ctx); plx.plx_timing_enable(ctx, True); plx.plx_timing_report(ctx)
    plx.plx_gcn_layer_bwd_chained(ctx, csr, False, X, dev(W), mask_src, dT, dev(Wn), saved, gdX, gdW, ws1, act=actc, order=order)
    launched = plx.plx_timing_report(ctx); plx.plx_timing_enable(ctx, False)
    # which path ran: the kernel that forms dF itself where the header says it does, one extra product elsewhere
    in_kernel = (dtype == "f32" and order == plx.PLX_ORDER_AGG_FIRST and 32 < din <= 128 and 64 < dout <= 128 and dn <= 32
                 and act != "values")
    assert any(name.endswith(f"fact{dn}") for name in launched) == in_kernel, launched
    plain = plx.plx_gcn_layer_workspace(csr, False, din, dout, dtype=code, act=actc, order=order)
    assert nbytes == plain if in_kernel else nbytes >= plain + m * dout * (4 if dtype == "f32" else 2)
    assert any(name.startswith("gemm_nt") and f"K{dn}]" in name for name in launched) == (not in_kernel), launched
    # unchained
    dF = matrix(m, dout); gdWn2 = torch.empty(dout, dn, device=DEV)
    plx.plx_gcn_layer_bwd(ctx, csr, True, F, dev(Wn), None, dZn, None, dF, gdWn2, ws2, act=plx.PLX_ACT_NONE,
                          order=plx.PLX_ORDER_COMBINE_FIRST)
    gdX2 = matrix(k, din); gdW2 = torch.empty(din, dout, device=DEV)
    plx.plx_gcn_layer_bwd(ctx, csr, False, X, dev(W), mask_src, dF, saved, gdX2, gdW2, ws1, act=actc, order=order)
    plx.plx_sync(ctx)
    F64 = F.double().cpu().numpy()
    dT64 = oracle.spmm_coo(m, row, c64, v64, dZn64)                       # (A^T)^T dZ'
    close(dT.float(), dT64, tol)
    close(gdWn, oracle.gemm(F64, dT64, ta=True), tol)
    assert torch.equal(gdWn, gdWn2)
    # the two GPU paths see the same mask and the same dT: they must agree closely everywhere
    agree = 2e-5 if dtype == "f32" else 2e-2                             # bf16: the unchained dF is rounded once more when stored
    assert rel_err(gdW, gdW2.double().cpu().numpy()) <= agree
    assert rel_err(gdX.float(), gdX2.double().cpu().numpy()) <= agree
    # against the oracle, from the stored dT (as both GPU paths take it) and with the mask decided where the GPU
    # decides it: the sign of its stored activation
    dQ = oracle.gemm(dT.double().cpu().numpy(), Wn, tb=True)
    if actc != plx.PLX_ACT_NONE:
        dQ = dQ * (F64 > 0)
    close(gdW, oracle.gemm(S, dQ, ta=True), tol)
    close(gdX.float(), oracle.spmm_t_coo(k, row, c64, v64, oracle.gemm(dQ, W, tb=True)), tol)
    close(F.float(), oracle.relu(Q) if actc != plx.PLX_ACT_NONE else Q, tol)
    if dtype == "f32":
        # end to end from the oracle's own values alone (no GPU tensor enters): Eq. 2.6 of the following layer, Eq. 2.4-2.7
        dQo = oracle.gemm(dT64, Wn, tb=True)
        if actc != plx.PLX_ACT_NONE:
            # Eq. 2.4: the oracle's own decision [Q > 0], except where it is ill-conditioned (|Q| within 1e-5 of zero):
            # there the decision is the kernel's, so that both sides differentiate the same function
            shaky = np.abs(Q) < BAND32 * np.abs(Q).max()
            assert (shaky & (Q != 0)).mean() < 1e-3                  # rows without entries give exact zeros: no decision there
            dQo = np.where(shaky, dQo * (F64 > 0), oracle.relu_bwd(Q, dQo))
        close(gdW, oracle.gemm(S, dQo, ta=True), tol)
        close(gdX, oracle.spmm_t_coo(k, row, c64, v64, oracle.gemm(dQo, W, tb=True)), tol)


@pytest.mark.parametrize("din,dout,dn,dtype,act", [
    (64, 128, 16, "f32", "bits"), (128, 128, 16, "f32", "values"), (100, 96, 7, "f32", "none"), (64, 64, 16, "f32", "bits"),
    (128, 33, 1, "f32", "values"),
    (32, 128, 16, "f32", "bits"), (64, 128, 17, "f32", "bits"), (602, 128, 16, "f32", "values"), (64, 128, 16, "bf16", "bits"),
    (64, 128, 16, "f32", "values-combine")])
def test_chained_forward_of_two_layers(ctx, din, dout, dn, dtype, act):
    """Forward of two consecutive layers where the first layer's last product also forms T = F Wn of the
    second (combine-first) layer, which then starts from T.  Shapes cover the kernel with the extra
    product (both tile widths, ragged widths, every activation form) and every fall-back (narrow or
    wide layer, dn above 16, bf16, combine-first first layer).  Against the oracle; F, the sign words
    and the saved aggregation must be bit-identical to the plain call's."""
    m, k = 1237, 1500
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    code = plx.PLX_F32 if dtype == "f32" else plx.PLX_BF16
    tol = TOL32 if dtype == "f32" else 2e-2
    order = plx.PLX_ORDER_COMBINE_FIRST if act.endswith("combine") else plx.PLX_ORDER_AGG_FIRST
    actc = {"bits": plx.PLX_ACT_RELU_BITS, "values": plx.PLX_ACT_RELU, "values-combine": plx.PLX_ACT_RELU, "none": plx.PLX_ACT_NONE}[act]
    rowptr, col, val = random_block(m, k, 7 * din + 3 * dout + dn)
    csr = plx.plx_csr_import(ctx, m, k, dev(rowptr), dev(col), dev(val))
    row, c64, v64 = coo_of(rowptr, col, val)
    r = np.random.default_rng(2 * din + dout + dn)

    def matrix(rows, cols, src=None, t=tdt, fill=0.0):       # rows padded to 16 bytes, as the network keeps them
        q = 16 // torch.empty(0, dtype=t).element_size()
        buf = torch.full((rows, -(-cols // q) * q), fill, dtype=t, device=DEV)
        if src is not None:
            buf[:, :cols] = torch.as_tensor(np.asarray(src, np.float32)).to(t).to(DEV)
        return buf, buf[:, :cols]

    _, X = matrix(k, din, r.standard_normal((k, din)))
    W = (r.standard_normal((din, dout)) * 0.2).astype(np.float32)
    Wn = (r.standard_normal((dout, dn)) * 0.2).astype(np.float32)
    X64 = X.double().cpu().numpy()
    Q = oracle.gemm(oracle.spmm_coo(m, row, c64, v64, X64), W)
    ws = torch.empty(plx.plx_gcn_layer_workspace(csr, False, din, dout, dtype=code, act=actc, order=order), dtype=torch.uint8, device=DEV)
    nw = (dout + 31) // 32
    outs = []
    for chained in (True, False):
        _, F = matrix(m, dout); _, saved = matrix(m, din)
        Tp, T = matrix(m, dn, fill=float("nan"))
        words = torch.zeros(m, nw, dtype=torch.int32, device=DEV)
        Zarg = words if actc == plx.PLX_ACT_RELU_BITS else None
        if chained:
            plx.plx_sync(ctx); plx.plx_timing_enable(ctx, True); plx.plx_timing_report(ctx)
            plx.plx_gcn_layer_fwd_chained(ctx, csr, False, X, dev(W), Zarg, F, saved, dev(Wn), T, ws, act=actc, order=order)
            launched = plx.plx_timing_report(ctx); plx.plx_timing_enable(ctx, False)
            in_kernel = (dtype == "f32" and order == plx.PLX_ORDER_AGG_FIRST and 32 < din <= 128 and din % 4 == 0
                         and 32 < dout <= 128 and dn <= 16)
            assert any(name.endswith(f"next{dn}") for name in launched) == in_kernel, launched
            assert any(f"N{dn},K{dout}]" in name for name in launched) == (not in_kernel), launched
        else:
            plx.plx_gcn_layer_fwd(ctx, csr, False, X, dev(W), Zarg, F, saved, ws, act=actc, order=order)
            plx.plx_gemm_nn(ctx, F, dev(Wn), T)
        _, Z2 = matrix(k, dn)
        plx.plx_gcn_layer_fwd_from_t(ctx, csr, True, T, Z2, None, act=plx.PLX_ACT_NONE)
        plx.plx_sync(ctx)
        outs.append((F, words, saved, T, Z2))
        F64 = F.double().cpu().numpy()
        close(F.float(), oracle.relu(Q) if actc != plx.PLX_ACT_NONE else Q, tol)
        T64 = oracle.gemm(F64, Wn)                                   # from the stored output, as the following layer sees it
        close(T.float(), T64, tol)
        assert bool(torch.isnan(Tp[:, dn:].float()).all())           # nothing written past dn
        close(Z2.float(), oracle.spmm_t_coo(k, row, c64, v64, T.double().cpu().numpy()), tol)
        if dtype == "f32":                                           # and from the oracle's own values alone
            To = oracle.gemm(oracle.relu(Q) if actc != plx.PLX_ACT_NONE else Q, Wn)
            close(T, To, tol)
            close(Z2, oracle.spmm_t_coo(k, row, c64, v64, To), tol)
    for a, b in zip(outs[0][:3], outs[1][:3]):
        assert torch.equal(a, b)
    assert rel_err(outs[0][3].float(), outs[1][3].double().cpu().numpy()) <= (2e-5 if dtype == "f32" else 2e-2)


def test_layer_pair_argument_errors(ctx):
    """Argument rules of the layer-pair calls that need a real adjacency handle."""
    m, k, din, dout, dn = 300, 400, 64, 128, 16
    rowptr, col, val = random_block(m, k, 77)
    csr = plx.plx_csr_import(ctx, m, k, dev(rowptr), dev(col), dev(val))
    X = torch.zeros(k, din, device=DEV); W = torch.zeros(din, dout, device=DEV); Wn = torch.zeros(dout, dn, device=DEV)
    F = torch.zeros(m, dout, device=DEV); saved = torch.zeros(m, din, device=DEV); T = torch.zeros(m, dn, device=DEV)
    dZn = torch.zeros(k, dn, device=DEV); gdX = torch.zeros(k, din, device=DEV)
    gdW = torch.zeros(din, dout, device=DEV); gdWn = torch.zeros(dout, dn, device=DEV)
    ws = torch.empty(plx.plx_gcn_layer_bwd_chained_workspace(ctx, csr, False, din, dout, dn, act=plx.PLX_ACT_NONE), dtype=torch.uint8, device=DEV)
    ws2 = torch.empty(plx.plx_gcn_layer_workspace(csr, True, dout, dn, act=plx.PLX_ACT_NONE, order=plx.PLX_ORDER_COMBINE_FIRST),
                      dtype=torch.uint8, device=DEV)

    def status(fn, *a, **kw):
        with pytest.raises(plx.PlxError) as e:
            fn(*a, **kw)
        return e.value.status

    # with an activation the following layer reads F: it must be given
    assert status(plx.plx_gcn_layer_fwd_chained, ctx, csr, False, X, W, torch.zeros(m, dout, device=DEV), None, saved, Wn, T, ws,
                  act=plx.PLX_ACT_RELU) == plx.PLX_ERR_INVALID
    # leading dimensions
    L = plx._lib
    h, c = ctx.handle, csr.handle
    assert L.plx_gcn_layer_fwd_chained(h, c, 0, X.data_ptr(), din, W.data_ptr(), dout, din, dout, 0, 0, 1, None, 0, F.data_ptr(), dout,
                                       saved.data_ptr(), din, Wn.data_ptr(), dn - 1, dn, T.data_ptr(), dn, ws.data_ptr(), ws.numel()) == plx.PLX_ERR_SHAPE
    assert L.plx_gcn_layer_fwd_chained(h, c, 0, X.data_ptr(), din, W.data_ptr(), dout, din, dout, 0, 0, 1, None, 0, F.data_ptr(), dout,
                                       saved.data_ptr(), din, Wn.data_ptr(), dn, 0, T.data_ptr(), dn, ws.data_ptr(), ws.numel()) == plx.PLX_ERR_INVALID
    assert L.plx_gcn_layer_fwd_from_t(h, c, 1, T.data_ptr(), dn - 1, dn, 0, 0, dZn.data_ptr(), dn, None, 0) == plx.PLX_ERR_SHAPE
    assert L.plx_gcn_layer_bwd_dt(h, c, 1, F.data_ptr(), dout, None, 0, dZn.data_ptr(), dn, dout, dn, 0, 0, T.data_ptr(), dn - 1,
                                  gdWn.data_ptr(), dn, ws2.data_ptr(), ws2.numel()) == plx.PLX_ERR_SHAPE
    assert L.plx_gcn_layer_bwd_dt(h, c, 1, F.data_ptr(), dout, None, 0, dZn.data_ptr(), dn, dout, dn, 0, 0, T.data_ptr(), dn,
                                  gdWn.data_ptr(), dn, ws2.data_ptr(), ws2.numel() - 1) == plx.PLX_ERR_SHAPE
    args = [h, c, 0, X.data_ptr(), din, W.data_ptr(), dout, None, 0, T.data_ptr(), dn, Wn.data_ptr(), dn, dn, saved.data_ptr(), din,
            din, dout, 0, 0, 1, gdX.data_ptr(), din, gdW.data_ptr(), dout, ws.data_ptr(), ws.numel()]
    assert L.plx_gcn_layer_bwd_chained(*args) == plx.PLX_OK
    bad = list(args); bad[10] = dn - 1                                       # lddtn < dn
    assert L.plx_gcn_layer_bwd_chained(*bad) == plx.PLX_ERR_SHAPE
    bad = list(args); bad[11] = None                                         # Wn
    assert L.plx_gcn_layer_bwd_chained(*bad) == plx.PLX_ERR_INVALID
    bad = list(args); bad[13] = 0                                            # dn
    assert L.plx_gcn_layer_bwd_chained(*bad) == plx.PLX_ERR_INVALID
    # unaligned rows of dT put the product outside the kernel: the workspace sized for the in-kernel path is then too small
    odd = torch.zeros(m, dn + 1, device=DEV)[:, :dn]
    bad = list(args); bad[9] = odd.data_ptr(); bad[10] = dn + 1
    assert L.plx_gcn_layer_bwd_chained(*bad) == plx.PLX_ERR_SHAPE
    assert b"smaller than" in L.plx_last_error(h)
    big = torch.empty(ws.numel() + m * dout * 4 + 256, dtype=torch.uint8, device=DEV)
    bad[-2] = big.data_ptr(); bad[-1] = big.numel()
    assert L.plx_gcn_layer_bwd_chained(*bad) == plx.PLX_OK
    plx.plx_sync(ctx)


def test_layer_very_wide_leading_dimension(ctx):
    """Rows 2^23 elements apart: the small-width dense kernels address a tile with 31-bit byte offsets
    and hand such matrices to the kernels with 64-bit addressing; results must not change."""
    m, k, din, dout, ld = 6, 7, 8, 12, 1 << 23
    rowptr, col, val = random_block(m, k, 9, empty_rows=False)
    csr = plx.plx_csr_import(ctx, m, k, dev(rowptr), dev(col), dev(val))
    row, c64, v64 = coo_of(rowptr, col, val)
    r = np.random.default_rng(4)
    X = r.standard_normal((k, din)).astype(np.float32)
    W = (r.standard_normal((din, dout)) * 0.3).astype(np.float32)
    dFn = r.standard_normal((m, dout)).astype(np.float32)
    Hagg = oracle.spmm_coo(m, row, c64, v64, X)
    Q = oracle.gemm(Hagg, W)
    dQ = oracle.relu_bwd(Q, dFn)
    dW = oracle.gemm(Hagg, dQ, ta=True)
    dX = oracle.spmm_t_coo(k, row, c64, v64, oracle.gemm(dQ, W, tb=True))

    def wide(rows, cols, src=None):
        t = torch.empty(rows, ld, device=DEV)[:, :cols]
        if src is not None:
            t.copy_(torch.as_tensor(src))
        return t

    for order in (plx.PLX_ORDER_AGG_FIRST, plx.PLX_ORDER_COMBINE_FIRST):
        ws = torch.empty(plx.plx_gcn_layer_workspace(csr, False, din, dout, order=order), dtype=torch.uint8, device=DEV)
        Xw, F, saved, dFw, gdX = wide(k, din, X), wide(m, dout), wide(m, din), wide(m, dout, dFn), wide(k, din)
        gdW = torch.empty(din, dout, device=DEV)
        plx.plx_gcn_layer_fwd(ctx, csr, False, Xw, dev(W), None, F, saved, ws, order=order)
        plx.plx_gcn_layer_bwd(ctx, csr, False, Xw, dev(W), F, dFw, saved, gdX, gdW, ws, order=order)
        plx.plx_sync(ctx)
        close(F, oracle.relu(Q), TOL32)
        close(gdW, dW, TOL32)
        close(gdX, dX, TOL32)
        del Xw, F, saved, dFw, gdX


@pytest.mark.parametrize("din,dout", [(64, 128), (128, 128), (100, 47), (128, 64), (36, 40), (128, 100)])
def test_split_products_switch(din, dout):
    """Wide fp32 layers go through six bf16 matrix products per fp32 product (three-way split of both
    operands) by default and through the fp32 matrix instructions when the switch is off: both must
    meet the fp32 tolerance against the oracle, and they must agree with each other far below it
    (the split drops only terms under 2^-23 of a product)."""
    m, k = 1500, 1300
    rowptr, col, val = random_block(m, k, 3 * din + dout)
    row, c64, v64 = coo_of(rowptr, col, val)
    r = np.random.default_rng(din + 11 * dout)
    X = r.standard_normal((k, din)).astype(np.float32)
    W = (r.standard_normal((din, dout)) * 0.2).astype(np.float32)
    Hagg = oracle.spmm_coo(m, row, c64, v64, X)
    Q = oracle.gemm(Hagg, W)
    dFn = (r.standard_normal((m, dout)) * (np.abs(Q) > BAND32 * np.abs(Q).max())).astype(np.float32)
    dQ = oracle.relu_bwd(Q, dFn)
    dW = oracle.gemm(Hagg, dQ, ta=True)
    dX = oracle.spmm_t_coo(k, row, c64, v64, oracle.gemm(dQ, W, tb=True))
    got = {}
    for on in (True, False):
        c = plx.plx_ctx(0)
        plx.plx_ctx_set_split_products(c, on)
        csr = plx.plx_csr_import(c, m, k, dev(rowptr), dev(col), dev(val))
        for order in (plx.PLX_ORDER_AGG_FIRST, plx.PLX_ORDER_COMBINE_FIRST):
            ws = torch.empty(plx.plx_gcn_layer_workspace(csr, False, din, dout, order=order), dtype=torch.uint8, device=DEV)
            F = torch.empty(m, dout, device=DEV); saved = torch.empty(m, din, device=DEV)
            gdX = torch.empty(k, din, device=DEV); gdW = torch.empty(din, dout, device=DEV)
            plx.plx_gcn_layer_fwd(c, csr, False, dev(X), dev(W), None, F, saved, ws, order=order)
            plx.plx_gcn_layer_bwd(c, csr, False, dev(X), dev(W), F, dev(dFn), saved, gdX, gdW, ws, order=order)
            plx.plx_sync(c)
            close(F, oracle.relu(Q), TOL32)
            close(gdW, dW, TOL32)
            close(gdX, dX, TOL32)
            got[(on, order)] = (F.cpu().numpy(), gdW.cpu().numpy(), gdX.cpu().numpy())
        csr.close(); c.close()
    for order in (plx.PLX_ORDER_AGG_FIRST, plx.PLX_ORDER_COMBINE_FIRST):
        for a, b in zip(got[(True, order)], got[(False, order)]):
            assert np.abs(a.astype(np.float64) - b).max() <= 2e-6 * np.abs(b).max()


@pytest.mark.parametrize("k", [64, 128])
def test_split_product_times_identity_is_exact(ctx, k):
    """A I = A bit for bit through the split path: the three bf16 parts of every element must add up
    to the element exactly (8 + 8 + 8 significand bits, each part rounded from what the others leave),
    over twenty decades of magnitude and both signs.  A lost or doubled bit anywhere in the split,
    the plane layout or the operand fragments shows up as a changed word."""
    m = 3001
    r = np.random.default_rng(k)
    A = (r.standard_normal((m, k)) * np.exp(r.uniform(-23, 23, (m, k)))).astype(np.float32)
    A[5, 7] = 0.0; A[6, 1] = -0.0; A[7, 3] = np.float32(1.0) + np.float32(2.0 ** -23); A[8, 2] = np.float32(16777215.0)
    big = np.finfo(np.float32).max                       # the largest finite values: their leading part must not round to infinity
    A[9, 0] = big; A[9, 1] = -big; A[10, 5] = np.nextafter(big, np.float32(0)); A[11, 4] = np.float32(3.39e38)
    eye = np.eye(k, dtype=np.float32)
    C = torch.empty(m, k, device=DEV)
    plx.plx_gemm_nn(ctx, dev(A), dev(eye), C); plx.plx_sync(ctx)
    g = C.cpu().numpy()
    assert np.array_equal(g.view(np.uint32)[A != 0], A.view(np.uint32)[A != 0])
    assert np.all(g[A == 0] == 0)


def test_split_products_extreme_and_non_finite_inputs():
    """The default fp32 path (three-way split into bf16 parts) on inputs the split could mishandle: finite values up to
    the largest fp32 number must give what the fp32 matrix instructions give (to rounding), with no NaN or infinity
    of the split's own making; an infinite or NaN input must make the same results non-finite in both paths."""
    m, K, N = 2000, 64, 128
    r = np.random.default_rng(9)
    A = r.standard_normal((m, K)).astype(np.float32)
    big = np.finfo(np.float32).max
    rows = r.choice(m, 200, replace=False)
    A[rows, r.integers(0, K, 200)] = (big * r.uniform(0.99, 1.0, 200) * r.choice([-1.0, 1.0], 200)).astype(np.float32)
    A[rows[0], :4] = [big, -big, np.nextafter(big, np.float32(0)), np.float32(2.0 ** 127)]
    W = (r.standard_normal((K, N)) * 1e-3).astype(np.float32)            # products stay finite
    ref = A.astype(np.float64) @ W.astype(np.float64)
    got = {}
    for on in (True, False):
        c = plx.plx_ctx(0)
        plx.plx_ctx_set_split_products(c, on)
        C = torch.empty(m, N, device=DEV)
        plx.plx_gemm_nn(c, dev(A), dev(W), C); plx.plx_sync(c)
        got[on] = C.cpu().numpy()
        assert np.isfinite(got[on]).all()
        # row by row: the huge entries dominate only their own rows
        err = np.abs(got[on] - ref).max(axis=1) / np.abs(ref).max(axis=1)
        assert err.max() <= 1e-5, (on, err.max())
        c.close()
    assert (np.abs(got[True].astype(np.float64) - got[False]).max(axis=1) / np.abs(ref).max(axis=1)).max() <= 2e-6
    bad = A.copy()
    bad[17, 3] = np.inf; bad[29, 60] = -np.inf; bad[41, 7] = np.nan
    for on in (True, False):
        c = plx.plx_ctx(0)
        plx.plx_ctx_set_split_products(c, on)
        C = torch.empty(m, N, device=DEV)
        plx.plx_gemm_nn(c, dev(bad), dev(W), C); plx.plx_sync(c)
        g = C.cpu().numpy()
        nonfinite_rows = np.nonzero(~np.isfinite(g).all(axis=1))[0]
        assert nonfinite_rows.tolist() == [17, 29, 41], (on, nonfinite_rows)
        assert not np.isfinite(g[[17, 29, 41]]).any()
        c.close()


def test_layer_seeded_sweep_of_shapes_layouts_and_modes(ctx):
    """120 seeded draws of (widths, block shape, dtype, order, activation mode, row padding): layer
    forward and backward against the oracle.  Widths sit on both sides of every tile and lane-group
    boundary, row paddings make aligned and unaligned layouts (padding holds NaN), the activation is
    none / ReLU with the value mask / ReLU with sign bits."""
    rng = np.random.default_rng(20250504)
    for case in range(120):
        din = int(rng.choice([1, 3, 8, 16, 31, 32, 33, 47, 64, 65, 96, 100, 127, 128]))
        dout = int(rng.choice([1, 4, 16, 17, 32, 40, 41, 64, 66, 100, 128]))
        m, k = int(rng.integers(1, 2500)), int(rng.integers(2, 2500))
        bf = bool(rng.integers(0, 2))
        tdt, code, tol = (torch.bfloat16, plx.PLX_BF16, 2e-2) if bf else (torch.float32, plx.PLX_F32, TOL32)
        order = int(rng.choice([plx.PLX_ORDER_AGG_FIRST, plx.PLX_ORDER_COMBINE_FIRST]))
        act = int(rng.choice([plx.PLX_ACT_NONE, plx.PLX_ACT_RELU, plx.PLX_ACT_RELU_BITS]))
        pad = int(rng.choice([0, 1, 8, 16]))
        tag = f"case {case}: {din}->{dout}, block {m}x{k}, bf16={bf}, order={order}, act={act}, pad={pad}"
        rowptr, col, val = random_block(m, k, case + 1000, empty_rows=m > 20)
        csr = plx.plx_csr_import(ctx, m, k, dev(rowptr), dev(col), dev(val))
        row, c64, v64 = coo_of(rowptr, col, val)

        def mat(a, width):
            ld = -(-width // pad) * pad if pad in (8, 16) else width + pad
            t = torch.full((a.shape[0], ld), float("nan"), dtype=tdt, device=DEV)
            t[:, :width] = torch.as_tensor(a.astype(np.float32)).to(tdt).to(DEV)
            return t, t[:, :width]

        _, X = mat(rng.standard_normal((k, din)), din)
        W = (rng.standard_normal((din, dout)) * 0.3).astype(np.float32)
        Hagg = oracle.spmm_coo(m, row, c64, v64, X.double().cpu().numpy())
        Q = oracle.gemm(Hagg, W)
        relu = act != plx.PLX_ACT_NONE
        Fref = oracle.relu(Q) if relu else Q
        keep = (np.abs(Q) > (3e-2 if bf else BAND32) * max(np.abs(Q).max(), 1e-30)) if relu else 1.0   # clear of the mask's rounding band
        _, dF = mat(rng.standard_normal((m, dout)) * keep, dout)
        dF64 = dF.double().cpu().numpy()
        dQ = oracle.relu_bwd(Q, dF64) if relu else dF64
        dW = oracle.gemm(Hagg, dQ, ta=True)
        dX = oracle.spmm_t_coo(k, row, c64, v64, oracle.gemm(dQ, W, tb=True))
        ws = torch.empty(plx.plx_gcn_layer_workspace(csr, False, din, dout, dtype=code, act=act, order=order), dtype=torch.uint8, device=DEV)
        (Fp, F), (_, saved), (gXp, gdX) = mat(np.zeros((m, dout)), dout), mat(np.zeros((m, din)), din), mat(np.zeros((k, din)), din)
        gdW = torch.empty(din, dout, device=DEV)
        Zm = torch.empty(m, (dout + 31) // 32, dtype=torch.int32, device=DEV) if act == plx.PLX_ACT_RELU_BITS else None
        plx.plx_gcn_layer_fwd(ctx, csr, False, X, dev(W), Zm, F, saved, ws, act=act, order=order)
        mask = Zm if act == plx.PLX_ACT_RELU_BITS else (F if relu else None)
        plx.plx_gcn_layer_bwd(ctx, csr, False, X, dev(W), mask, dF, saved, gdX, gdW, ws, act=act, order=order)
        plx.plx_sync(ctx)
        for name, g, o in (("F", F, Fref), ("dW", gdW, dW), ("dX", gdX, dX)):
            err = np.abs(g.double().cpu().numpy() - o).max() / max(np.abs(o).max(), 1e-30)
            assert err <= tol, f"{tag}: {name} off by {err:.3e}"
        for t, width in ((Fp, dout), (gXp, din)):                          # padding untouched
            assert bool(torch.isnan(t[:, width:].float()).all()), tag
        csr.close()


def test_layer_sign_bits_argument_errors(ctx):
    m, k, din, dout = 40, 50, 8, 40
    rowptr, col, val = random_block(m, k, 2)
    csr = plx.plx_csr_import(ctx, m, k, dev(rowptr), dev(col), dev(val))
    X = torch.zeros(k, din, device=DEV); W = torch.zeros(din, dout, device=DEV)
    F = torch.empty(m, dout, device=DEV); saved = torch.empty(m, din, device=DEV)
    words = torch.empty(m, 2, dtype=torch.int32, device=DEV)
    # two words per row by shape, but rows only one word apart: the binding sees a large enough tensor, the library a
    # leading dimension below the two words that 40 columns need
    one_word = torch.empty(m + 1, dtype=torch.int32, device=DEV).as_strided((m, 2), (1, 1))
    ws = torch.empty(plx.plx_gcn_layer_workspace(csr, False, din, dout, act=plx.PLX_ACT_RELU_BITS), dtype=torch.uint8, device=DEV)
    bits_act = plx.PLX_ACT_RELU_BITS
    with pytest.raises(ValueError, match="Z: shape"):                          # too few words per row by shape: the binding's check
        plx.plx_gcn_layer_fwd(ctx, csr, False, X, W, torch.empty(m, 1, dtype=torch.int32, device=DEV), F, saved, ws, act=bits_act)
    with pytest.raises(plx.PlxError) as err:                                   # unknown activation code
        plx.plx_gcn_layer_fwd(ctx, csr, False, X, W, words, F, saved, ws, act=3)
    assert err.value.status == plx.PLX_ERR_INVALID
    with pytest.raises(plx.PlxError) as err:                                   # the words go beside F, not instead of it
        plx.plx_gcn_layer_fwd(ctx, csr, False, X, W, words, None, saved, ws, act=bits_act)
    assert err.value.status == plx.PLX_ERR_INVALID
    with pytest.raises(plx.PlxError) as err:                                   # 40 columns need two words per row
        plx.plx_gcn_layer_fwd(ctx, csr, False, X, W, one_word, F, saved, ws, act=bits_act)
    assert err.value.status == plx.PLX_ERR_SHAPE
    dX = torch.empty(k, din, device=DEV); dW = torch.empty(din, dout, device=DEV)
    with pytest.raises(plx.PlxError) as err:
        plx.plx_gcn_layer_bwd(ctx, csr, False, X, W, None, F, saved, dX, dW, ws, act=bits_act)
    assert err.value.status == plx.PLX_ERR_INVALID
    with pytest.raises(plx.PlxError) as err:
        plx.plx_gcn_layer_bwd(ctx, csr, False, X, W, one_word, F, saved, dX, dW, ws, act=bits_act)
    assert err.value.status == plx.PLX_ERR_SHAPE


def test_network_step_in_hip_graph():
    """One whole forward + backward of configs[0] recorded into a HIP graph: every replay, with
    eager work and synchronisations in between, reproduces the eager step bit for bit (the
    kernels are deterministic; the recorded step holds no memset node and allocates nothing)."""
    from paper_2505_04083_amd.network import GcnNetwork
    cfg = synth.CONFIGS["tiny"]
    side = torch.cuda.Stream(device=DEV)
    gctx = plx.plx_ctx(0, stream=side.cuda_stream)
    src, dst = cfg.edges(DEV)
    pr, pc = cfg.perms(DEV)
    H0 = cfg.features(DEV); Ws = cfg.weights(DEV); y = cfg.labels(DEV)
    torch.cuda.synchronize()
    csr = plx.plx_build_csr(gctx, cfg.n, src, dst, pr, pc)
    net = GcnNetwork(gctx, csr, Ws)
    net.step(H0, y); net.sync()
    want = [w.clone() for w in net.dW] + [net.dH[0].clone(), net.loss.clone()]
    graph = net.capture(H0, y, side)
    for rep in range(4):
        for t in net.dW + [net.dH[0], net.loss]:
            t.fill_(float("nan"))                                   # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = net.dW + [net.dH[0], net.loss]
        for g, w in zip(got, want):
            assert torch.equal(g, w), f"replay {rep} differs from the eager step"
        if rep == 1:                                                # an eager step between replays
            net.step(H0, y); net.sync()
    del graph
    csr.close(); gctx.close()


def test_first_step_recorded_into_a_hip_graph_without_an_eager_one():
    """A step allocates nothing and never waits -- the partial sums of split rows live in the adjacency handle -- so the
    very first step of a network can be recorded into a HIP graph (no eager step before it to size any buffer).  Graph
    with rows far above the segment threshold (social recipe); the replays must equal the eager step that follows."""
    from paper_2505_04083_amd.network import GcnNetwork
    cfg = synth.CONFIGS["social"].scaled(0.05)
    cfg.dims = [64, 128, 128, 41]
    side = torch.cuda.Stream(device=DEV)
    gctx = plx.plx_ctx(0, stream=side.cuda_stream)
    src, dst = cfg.edges(DEV)
    pr, pc = cfg.perms(DEV)
    H0 = cfg.features(DEV); Ws = cfg.weights(DEV); y = cfg.labels(DEV)
    torch.cuda.synchronize()
    csr = plx.plx_build_csr(gctx, cfg.n, src, dst, pr, pc)
    assert plx.plx_csr_bins(csr, False)[0][1] + plx.plx_csr_bins(csr, False)[0][2] > 100     # rows that go through segments
    net = GcnNetwork(gctx, csr, Ws)
    live = len(gctx._live)
    graph = net.capture(H0, y, side)
    assert len(gctx._live) == live                                  # recording obtained nothing from the allocator
    got = []
    for rep in range(2):
        for t in net.dW + [net.dH[0], net.loss]:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got.append([t.clone() for t in net.dW + [net.dH[0], net.loss]])
    net.step(H0, y); net.sync()
    for g in got:
        for a, b in zip(g, net.dW + [net.dH[0], net.loss]):
            assert torch.equal(a, b)
    del graph
    csr.close(); gctx.close()


# ---------------------------------------------------------------- bf16 storage, fp32 accumulation
TOLBF = 2e-2


def fro_err(gpu, ref):
    g = gpu.detach().double().cpu().numpy()
    return float(np.linalg.norm(g - ref) / np.linalg.norm(ref))


def bf(a):
    """fp32 array -> (bf16 device tensor, the same values widened back to fp64 for the oracle)."""
    t = torch.as_tensor(np.asarray(a, np.float32)).to(torch.bfloat16)
    return t.to(DEV).contiguous(), t.double().numpy()


@pytest.mark.parametrize("d,pad", [(32, 0), (128, 0), (47, 1), (41, 0), (100, 4), (300, 4)])
def test_spmm_bf16_parity(ctx, d, pad):
    m, k = 1531, 9973
    rowptr, col, val = random_block(m, k, 31 + d, giant_row=70)
    csr = plx.plx_csr_import(ctx, m, k, dev(rowptr), dev(col), dev(val))
    row, c64, v64 = coo_of(rowptr, col, val)
    r = np.random.default_rng(d)
    Xd, X64 = bf(r.standard_normal((k, d)))
    Gd, G64 = bf(r.standard_normal((m, d)))
    ld = d + pad
    Xp = torch.zeros(k, ld, dtype=torch.bfloat16, device=DEV); Xp[:, :d] = Xd
    Gp = torch.zeros(m, ld, dtype=torch.bfloat16, device=DEV); Gp[:, :d] = Gd
    Y = torch.zeros(m, ld, dtype=torch.bfloat16, device=DEV)
    Yt = torch.zeros(k, ld, dtype=torch.bfloat16, device=DEV)
    plx.plx_spmm(ctx, csr, Xp[:, :d], Y[:, :d]); plx.plx_spmm_t(ctx, csr, Gp[:, :d], Yt[:, :d]); plx.plx_sync(ctx)
    assert rel_err(Y[:, :d], oracle.spmm_coo(m, row, c64, v64, X64)) <= TOLBF
    assert rel_err(Yt[:, :d], oracle.spmm_t_coo(k, row, c64, v64, G64)) <= TOLBF


@pytest.mark.parametrize("din,dout", [(32, 128), (128, 128), (100, 47), (128, 16), (64, 128), (40, 72)])
def test_layer_bf16_both_orders(ctx, din, dout):
    """One layer with bf16 activations / gradients (fp32 weights, fp32 accumulation, fp32 dW);
    the oracle sees the same bf16-rounded inputs in fp64."""
    m, k = 1300, 1700
    rowptr, col, val = random_block(m, k, 3 * din + dout)
    csr = plx.plx_csr_import(ctx, m, k, dev(rowptr), dev(col), dev(val))
    row, c64, v64 = coo_of(rowptr, col, val)
    r = np.random.default_rng(din + dout)
    Xd, X64 = bf(r.standard_normal((k, din)))
    W = (r.standard_normal((din, dout)) * 0.2).astype(np.float32)
    dFd, dF64 = bf(r.standard_normal((m, dout)))
    Hagg = oracle.spmm_coo(m, row, c64, v64, X64)
    Q = oracle.gemm(Hagg, W)
    # the GPU takes the mask from its own bf16 activation; keep clear of the rounding band
    dF64 = dF64 * (np.abs(Q) > 2e-2 * np.abs(Q).max())
    dFd = torch.as_tensor(dF64.astype(np.float32)).to(torch.bfloat16).to(DEV)
    dQ = oracle.relu_bwd(Q, dF64)
    dW = oracle.gemm(Hagg, dQ, ta=True)
    dX = oracle.spmm_t_coo(k, row, c64, v64, oracle.gemm(dQ, W, tb=True))
    for order in (plx.PLX_ORDER_AGG_FIRST, plx.PLX_ORDER_COMBINE_FIRST):
        nbytes = plx.plx_gcn_layer_workspace(csr, False, din, dout, dtype=plx.PLX_BF16, order=order)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
        F = torch.empty(m, dout, dtype=torch.bfloat16, device=DEV)
        saved = torch.empty(m, din, dtype=torch.bfloat16, device=DEV)
        plx.plx_gcn_layer_fwd(ctx, csr, False, Xd, dev(W), None, F, saved, ws, order=order)
        gdX = torch.empty(k, din, dtype=torch.bfloat16, device=DEV); gdW = torch.empty(din, dout, device=DEV)
        plx.plx_gcn_layer_bwd(ctx, csr, False, Xd, dev(W), F, dFd, saved, gdX, gdW, ws, order=order)
        plx.plx_sync(ctx)
        assert rel_err(F, oracle.relu(Q)) <= TOLBF
        assert rel_err(gdW, dW) <= TOLBF
        assert rel_err(gdX, dX) <= TOLBF


@pytest.mark.parametrize("din,dout", [(602, 128), (200, 150), (96, 200), (301, 41)])
def test_layer_bf16_wide_widths_on_aligned_rows(ctx, din, dout):
    """bf16 layers with a width above 128 (the 602-feature input layer of the social workload): the
    separate dense products on 16-byte aligned rows, both orders, with the ReLU mask as values."""
    m, k = 1300, 1700
    rowptr, col, val = random_block(m, k, 7 * din + dout)
    csr = plx.plx_csr_import(ctx, m, k, dev(rowptr), dev(col), dev(val))
    row, c64, v64 = coo_of(rowptr, col, val)
    r = np.random.default_rng(din + 2 * dout)

    def rows16(a):
        ld = -(-a.shape[1] // 8) * 8
        t = torch.full((a.shape[0], ld), float("nan"), dtype=torch.bfloat16, device=DEV)
        t[:, :a.shape[1]] = torch.as_tensor(np.asarray(a, np.float32)).to(torch.bfloat16).to(DEV)
        return t, t[:, :a.shape[1]]

    _, Xd = rows16(r.standard_normal((k, din)))
    X64 = Xd.double().cpu().numpy()
    W = (r.standard_normal((din, dout)) * 0.2).astype(np.float32)
    Hagg = oracle.spmm_coo(m, row, c64, v64, X64)
    Q = oracle.gemm(Hagg, W)
    dF = r.standard_normal((m, dout)) * (np.abs(Q) > 2e-2 * np.abs(Q).max())      # keep clear of the mask's rounding band
    _, dFd = rows16(dF)
    dF64 = dFd.double().cpu().numpy()
    dQ = oracle.relu_bwd(Q, dF64)
    dW = oracle.gemm(Hagg, dQ, ta=True)
    dX = oracle.spmm_t_coo(k, row, c64, v64, oracle.gemm(dQ, W, tb=True))
    for order in (plx.PLX_ORDER_AGG_FIRST, plx.PLX_ORDER_COMBINE_FIRST):
        nbytes = plx.plx_gcn_layer_workspace(csr, False, din, dout, dtype=plx.PLX_BF16, order=order)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
        Fp, F = rows16(np.zeros((m, dout)))
        _, saved = rows16(np.zeros((m, din)))
        gXp, gdX = rows16(np.zeros((k, din)))
        gdW = torch.empty(din, dout, device=DEV)
        plx.plx_gcn_layer_fwd(ctx, csr, False, Xd, dev(W), None, F, saved, ws, order=order)
        plx.plx_gcn_layer_bwd(ctx, csr, False, Xd, dev(W), F, dFd, saved, gdX, gdW, ws, order=order)
        plx.plx_sync(ctx)
        assert rel_err(F.float(), oracle.relu(Q)) <= TOLBF
        assert rel_err(gdW, dW) <= TOLBF
        assert rel_err(gdX.float(), dX) <= TOLBF
        for t, wdt in ((Fp, dout), (gXp, din)):                                  # padding untouched
            assert bool(torch.isnan(t[:, wdt:].float()).all())


def test_three_layer_network_bf16(ctx):
    """configs[0] with bf16 storage end to end, held to the bf16 tolerance (2e-2, max norm) on the logits, the
    loss and EVERY gradient tensor.  The sign of a pre-activation (Eq. 2.4) is an integer decision: the GPU takes
    it from its stored bf16 activation, which differs from the fp64 one by ~2^-9 of its scale, so about that
    share of the decisions differ from the oracle's own and each one moves a gradient entry by a whole term.
    Both sides therefore take the decision in the kernel's precision: the oracle's backward pass is handed the
    masks [F > 0] of the GPU's stored activations.  Against the oracle's own decisions the gradients are
    still close as vectors (1e-1 in the Frobenius norm)."""
    cfg = synth.CONFIGS["tiny"]
    src, dst = cfg.edges()
    pr, pc = cfg.perms()
    F0 = cfg.features().to(torch.bfloat16)
    Ws, y = cfg.weights(), cfg.labels()
    adj = oracle.adjacency(cfg.n, src.numpy(), dst.numpy())
    Wn = [w.numpy() for w in Ws]
    ref = ogcn.forward_backward(adj, F0.double().numpy(), Wn, y.numpy())
    csr = plx.plx_build_csr(ctx, cfg.n, src.to(DEV), dst.to(DEV), pr.to(DEV), pc.to(DEV))
    H0 = torch.empty_like(F0); H0[pc] = F0
    y_gpu = torch.empty_like(y); y_gpu[pr] = y
    run = run_network(ctx, csr, H0.to(DEV), [w.to(DEV) for w in Ws], y_gpu.to(DEV))
    assert rel_err(run.Z[-1][pr.to(DEV)], ref.logits) <= TOLBF
    assert abs(run.loss.item() - ref.loss) / ref.loss <= TOLBF
    for l in range(len(Ws)):
        assert fro_err(run.dW[l], ref.dW[l]) <= 1e-1, f"dW of layer {l}"
    assert fro_err(run.dF0[pc.to(DEV)], ref.dF[0]) <= 1e-1
    # the kernel's decisions: layer l's output is in P_r order for even l, in P_c order for odd l (Eq. 5.3-5.4)
    masks = []
    for l in range(len(Ws) - 1):
        perm = (pr if l % 2 == 0 else pc).to(DEV)
        masks.append((run.F[l][perm].float() > 0).cpu().numpy())
    flipped = np.mean([(m != (q > 0)).mean() for m, q in zip(masks, ref.Q)])
    assert 0 < flipped < 2e-2                                            # a small share of decisions differs, as expected
    same = ogcn.forward_backward(adj, F0.double().numpy(), Wn, y.numpy(), masks=masks + [None])
    for l in range(len(Ws)):
        assert rel_err(run.dW[l], same.dW[l]) <= TOLBF, f"dW of layer {l}"
    assert rel_err(run.dF0[pc.to(DEV)].float(), same.dF[0]) <= TOLBF


def test_allocator_failure_is_reported_and_leaks_nothing():
    """Every device allocation of the two set-up calls fails in turn (the context's allocator hook returns NULL from the
    k-th request on): the call must return PLX_ERR_OOM, hand out no handle, and give back everything it had obtained."""
    import ctypes
    L = plx._lib
    live, state = {}, {"n": 0, "fail_from": None}

    def alloc(nbytes, _user):
        state["n"] += 1
        if state["fail_from"] is not None and state["n"] > state["fail_from"]:
            return None
        t = torch.empty(max(int(nbytes), 1), dtype=torch.uint8, device=DEV)
        live[t.data_ptr()] = t
        return t.data_ptr()

    def free(p, _user):
        assert p in live, "freed a pointer the allocator never handed out (or freed it twice)"
        del live[p]

    a_cb, f_cb = plx._ALLOC_FN(alloc), plx._FREE_FN(free)
    h = ctypes.c_void_p()
    assert L.plx_ctx_create(0, torch.cuda.current_stream().cuda_stream, a_cb, f_cb, None, ctypes.byref(h)) == plx.PLX_OK
    m, k = 700, 3000
    rowptr, col, val = random_block(m, k, 5, giant_row=9)
    rp, c, v = dev(rowptr), dev(col), dev(val)
    cfg = synth.CONFIGS["tiny"].scaled(0.25)
    src, dst = (t.to(DEV) for t in cfg.edges())
    pr, pc = (t.to(DEV) for t in cfg.perms())
    calls = {
        "plx_csr_import": lambda out: L.plx_csr_import(h, m, k, len(col), rp.data_ptr(), c.data_ptr(), v.data_ptr(), ctypes.byref(out)),
        "plx_build_csr": lambda out: L.plx_build_csr(h, cfg.n, src.numel(), src.data_ptr(), dst.data_ptr(), pr.data_ptr(), pc.data_ptr(),
                                                    ctypes.byref(out)),
    }
    for name, call in calls.items():
        state.update(n=0, fail_from=None)
        out = ctypes.c_void_p()
        assert call(out) == plx.PLX_OK and out.value
        total = state["n"]
        assert total >= 5 and len(live) > 0
        L.plx_csr_destroy(h, out)
        assert not live, f"{name}: {len(live)} buffers still held after the handle was destroyed"
        for fail_from in range(total):
            state.update(n=0, fail_from=fail_from)
            out = ctypes.c_void_p()
            st = call(out)
            assert st == plx.PLX_ERR_OOM, f"{name}: allocation {fail_from + 1} of {total} failed, status {st}"
            assert not out.value and b"allocation" in L.plx_last_error(h)
            assert not live, f"{name}: {len(live)} buffers leaked when allocation {fail_from + 1} of {total} failed"
    L.plx_ctx_destroy(h)
    assert not live


@pytest.mark.parametrize("din,dout,act", [(32, 128, "bits"), (32, 128, "relu"), (20, 47, "bits"), (32, 16, "none"), (17, 100, "relu"),
                                          (24, 96, "bits")])
def test_fused_aggregation_forward(din, dout, act):
    """Aggregate-first forward with Eq. 2.2-2.3 in the epilogue of the sparse kernels (plx_ctx_set_fused_aggregation):
    both row bins (lane-group rows, and rows summed from segments with the row-list epilogue), empty rows, a partial
    last tile; against the oracle, and against the separate kernels (H bit-identical, results to rounding, sign words
    exactly the packed [F > 0]); the backward call then runs on what the fused forward left."""
    m, k = 1237, 3000
    rowptr, col, val = random_block(m, k, 5 * din + dout, giant_row=33)
    row, c64, v64 = coo_of(rowptr, col, val)
    r = np.random.default_rng(din * dout)
    X = r.standard_normal((k, din)).astype(np.float32)
    W = (r.standard_normal((din, dout)) * 0.3).astype(np.float32)
    Hagg = oracle.spmm_coo(m, row, c64, v64, X)
    Q = oracle.gemm(Hagg, W)
    actc = {"bits": plx.PLX_ACT_RELU_BITS, "relu": plx.PLX_ACT_RELU, "none": plx.PLX_ACT_NONE}[act]
    dF = (r.standard_normal((m, dout)) * (np.abs(Q) > BAND32 * np.abs(Q).max())).astype(np.float32)
    dQ = oracle.relu_bwd(Q, dF) if act != "none" else dF.astype(np.float64)
    nw = (dout + 31) // 32
    got = {}
    for fused in (True, False):
        c = plx.plx_ctx(0)
        plx.plx_ctx_set_fused_aggregation(c, fused)
        csr = plx.plx_csr_import(c, m, k, dev(rowptr), dev(col), dev(val))
        (sub, wave, split), _ = plx.plx_csr_bins(csr, False)
        assert sub > 0 and wave + split > 0
        ws = torch.empty(plx.plx_gcn_layer_workspace(csr, False, din, dout, act=actc, order=plx.PLX_ORDER_AGG_FIRST), dtype=torch.uint8, device=DEV)
        ld = -(-din // 4) * 4                                             # rows padded to 16 bytes, the padding holds NaN
        Xd = torch.full((k, ld), float("nan"), device=DEV)[:, :din]; Xd.copy_(dev(X))
        F = torch.full((m, dout), 7.0, device=DEV); saved = torch.full((m, ld), float("nan"), device=DEV)[:, :din]
        words = torch.full((m, nw), 0x5A5A5A5A, dtype=torch.int32, device=DEV)
        plx.plx_timing_enable(c, True); plx.plx_timing_report(c)
        plx.plx_gcn_layer_fwd(c, csr, False, Xd, dev(W), words if act == "bits" else None, F, saved, ws, act=actc,
                              order=plx.PLX_ORDER_AGG_FIRST)
        launched = plx.plx_timing_report(c); plx.plx_timing_enable(c, False)
        assert any(n.startswith("spmm_subwave_combine") for n in launched) == fused, launched
        assert any(n.startswith("rows_combine") for n in launched) == fused, launched
        close(saved, Hagg, TOL32)
        close(F, oracle.relu(Q) if act != "none" else Q, TOL32)
        if act == "bits":
            pos = (F > 0).cpu().numpy()
            padded = np.zeros((m, 32 * nw), dtype=np.uint64); padded[:, :dout] = pos
            want = (padded.reshape(m, nw, 32) << np.arange(32, dtype=np.uint64)).sum(axis=2).astype(np.uint32)
            assert np.array_equal(words.cpu().numpy().view(np.uint32), want)
        gdX = torch.empty(k, din, device=DEV); gdW = torch.empty(din, dout, device=DEV)
        mask = {"bits": words, "relu": F, "none": None}[act]
        plx.plx_gcn_layer_bwd(c, csr, False, Xd, dev(W), mask, dev(dF), saved, gdX, gdW, ws, act=actc, order=plx.PLX_ORDER_AGG_FIRST)
        plx.plx_sync(c)
        close(gdW, oracle.gemm(Hagg, dQ, ta=True), TOL32)
        close(gdX, oracle.spmm_t_coo(k, row, c64, v64, oracle.gemm(dQ, W, tb=True)), TOL32)
        got[fused] = (saved.cpu().numpy(), F.cpu().numpy())
        csr.close(); c.close()
    assert np.array_equal(got[True][0], got[False][0])                    # the aggregation itself: same kernel code, same bits
    assert np.abs(got[True][1].astype(np.float64) - got[False][1]).max() <= 2e-6 * np.abs(got[False][1]).max()


def test_layers_on_an_adjacency_without_entries_or_without_nodes(ctx):
    """A block with rows and columns but no stored entry: A H = 0, so the forward outputs (values, sign words, the
    aggregation, the following layer's T) are zero and so is every gradient; nothing is launched with an empty grid.
    A graph without nodes: the layer calls succeed and dW is zero."""
    m, k, din, dout, dn = 5, 7, 64, 128, 16
    csr = plx.plx_csr_import(ctx, m, k, dev(np.zeros(m + 1, np.int64)), dev(np.zeros(0, np.int32)), dev(np.zeros(0, np.float32)))
    for order in (plx.PLX_ORDER_AGG_FIRST, plx.PLX_ORDER_COMBINE_FIRST):
        H = torch.randn(k, din, device=DEV); W = torch.randn(din, dout, device=DEV); Wn = torch.randn(dout, dn, device=DEV)
        ws = torch.empty(max(1, plx.plx_gcn_layer_bwd_chained_workspace(ctx, csr, False, din, dout, dn, act=plx.PLX_ACT_RELU_BITS, order=order)),
                         dtype=torch.uint8, device=DEV)
        F = torch.full((m, dout), 7.0, device=DEV); saved = torch.full((m, din), 7.0, device=DEV); T = torch.full((m, dn), 7.0, device=DEV)
        words = torch.full((m, 4), 0x5A5A5A5A, dtype=torch.int32, device=DEV)
        plx.plx_gcn_layer_fwd_chained(ctx, csr, False, H, W, words, F, saved, Wn, T, ws, act=plx.PLX_ACT_RELU_BITS, order=order)
        plx.plx_sync(ctx)
        assert float(F.abs().max()) == 0 and float(T.abs().max()) == 0 and int(words.abs().max()) == 0
        if order == plx.PLX_ORDER_AGG_FIRST:
            assert float(saved.abs().max()) == 0
        dH = torch.full((k, din), 7.0, device=DEV); dW = torch.full((din, dout), 7.0, device=DEV)
        plx.plx_gcn_layer_bwd(ctx, csr, False, H, W, words, torch.randn(m, dout, device=DEV), saved, dH, dW, ws, act=plx.PLX_ACT_RELU_BITS, order=order)
        plx.plx_sync(ctx)
        assert float(dH.abs().max()) == 0 and float(dW.abs().max()) == 0
    Y = torch.full((m, 8), 7.0, device=DEV)
    plx.plx_spmm(ctx, csr, torch.randn(k, 8, device=DEV), Y); plx.plx_sync(ctx)
    assert float(Y.abs().max()) == 0
    csr.close()
    e = torch.zeros(0, dtype=torch.int64, device=DEV)
    none = plx.plx_build_csr(ctx, 0, e, e)
    assert none.nnz == 0 and none.m == 0
    W = torch.randn(din, dout, device=DEV); dW = torch.full((din, dout), 7.0, device=DEV)
    z = lambda c, t=torch.float32: torch.empty(0, c, dtype=t, device=DEV)
    ws = torch.empty(256, dtype=torch.uint8, device=DEV)
    plx.plx_gcn_layer_fwd(ctx, none, False, z(din), W, None, z(dout), z(din), ws)
    plx.plx_gcn_layer_bwd(ctx, none, False, z(din), W, z(dout), z(dout), z(din), z(din), dW, ws)
    plx.plx_sync(ctx)
    assert float(dW.abs().max()) == 0
    none.close()
