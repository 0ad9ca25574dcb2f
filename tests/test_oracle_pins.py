"""Pins for the CPU oracle: every oracle function is checked against something other than
itself -- closed forms, invariants, a dense numpy brute force, finite differences and the
values the paper prints (tests/golden).  CPU only."""
import math
import os

import numpy as np
import pytest

import oracle
from oracle import dense as odense
from oracle import gcn as ogcn
import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(1234)


def small_graph(n=48, e=160, seed=7):
    r = np.random.default_rng(seed)
    src = r.integers(0, n, e)
    dst = r.integers(0, n, e)
    return n, src, dst


def to_dense(adj):
    A = np.zeros((adj.n, adj.n))
    A[adj.row, adj.col] = adj.val
    return A


def read_table(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append(line.split())
    return rows


# ---------------------------------------------------------------- adjacency (Sec. 2.1)

def test_structure_rule_matches_table4():
    """Table 4: nonzeros = 2*edges + nodes exactly for Reddit, Isolate-3-8M, europe_osm --
    the rule the oracle implements (symmetrise, dedupe, one loop per node)."""
    t = {r[0]: list(map(int, r[1:])) for r in read_table("table4_datasets.txt")}
    for name in ("Reddit", "Isolate-3-8M", "europe_osm"):
        n, e, nnz = t[name][:3]
        assert 2 * e + n == nnz
    # and the oracle reproduces the rule on a graph with duplicates, loops, both directions
    n, src, dst = small_graph()
    src = np.concatenate([src, dst[:20], np.arange(5)])     # reversed copies + self-loops
    dst = np.concatenate([dst, src[:20], np.arange(5)])
    uniq = {(min(u, v), max(u, v)) for u, v in zip(src.tolist(), dst.tolist()) if u != v}
    adj = oracle.adjacency(n, src, dst)
    assert adj.nnz == 2 * len(uniq) + n
    assert adj.deg.sum() == adj.nnz
    # sorted by (row, col), no duplicates
    key = adj.row * n + adj.col
    assert np.all(np.diff(key) > 0)


def test_adjacency_invariants():
    n, src, dst = small_graph(64, 300, 3)
    adj = oracle.adjacency(n, src, dst)
    A = to_dense(adj)
    assert np.array_equal(A, A.T)                                  # symmetric, bit-equal
    assert np.all(adj.val > 0) and np.all(adj.val <= 1)
    assert np.allclose(np.diag(A), 1.0 / adj.deg, rtol=0, atol=1e-16)   # diag = 1/d_u
    s = np.sqrt(adj.deg.astype(np.float64))
    assert np.allclose(A @ s, s, rtol=1e-13)                       # eigenvector sqrt(d), eigenvalue 1
    # independent dense construction
    A2, d2 = odense.dense_adjacency(n, src, dst)
    assert np.array_equal(d2, adj.deg)
    assert np.allclose(A, A2, rtol=1e-15, atol=0)


def test_isolated_node_and_empty_graph():
    adj = oracle.adjacency(5, np.array([0]), np.array([1]))
    A = to_dense(adj)
    assert A[4, 4] == 1.0 and A[0, 0] == 0.5 and A[0, 1] == 0.5
    adj0 = oracle.adjacency(6, np.zeros(0, np.int64), np.zeros(0, np.int64))
    assert np.array_equal(to_dense(adj0), np.eye(6))
    with pytest.raises(ValueError):
        oracle.adjacency(3, np.array([0]), np.array([3]))


def test_closed_form_graphs():
    n = 9
    # complete graph: A^ = J/n
    iu = np.triu_indices(n, 1)
    A = to_dense(oracle.adjacency(n, iu[0], iu[1]))
    assert np.allclose(A, np.full((n, n), 1.0 / n), rtol=1e-15)
    # ring: every entry 1/3 on the tridiagonal-with-wrap pattern
    r = np.arange(n)
    A = to_dense(oracle.adjacency(n, r, (r + 1) % n))
    expect = np.zeros((n, n))
    for i in range(n):
        for j in (i - 1, i, i + 1):
            expect[i, j % n] = 1.0 / 3.0
    assert np.allclose(A, expect, rtol=1e-15)
    # star: hub 0 with n-1 leaves
    A = to_dense(oracle.adjacency(n, np.zeros(n - 1, np.int64), np.arange(1, n)))
    assert math.isclose(A[0, 0], 1.0 / n) and math.isclose(A[1, 1], 0.5)
    assert math.isclose(A[0, 3], 1.0 / math.sqrt(2 * n)) and A[1, 2] == 0.0
    # single edge
    A = to_dense(oracle.adjacency(2, np.array([0]), np.array([1])))
    assert np.array_equal(A, np.full((2, 2), 0.5))


# ---------------------------------------------------------------- sparse and dense products

def test_spmm_matches_dense_and_adjoint():
    n, src, dst = small_graph(40, 150, 11)
    adj = oracle.adjacency(n, src, dst)
    A = to_dense(adj)
    # make it non-symmetric in values so a transposed operand would be caught
    val = adj.val * (1.0 + 0.1 * np.sin(adj.row * 3.0 + adj.col * 7.0))
    A = np.zeros((n, n)); A[adj.row, adj.col] = val
    X = rng.standard_normal((n, 5)); Y = rng.standard_normal((n, 5))
    AX = oracle.spmm_coo(n, adj.row, adj.col, val, X)
    ATY = oracle.spmm_t_coo(n, adj.row, adj.col, val, Y)
    assert np.allclose(AX, A @ X, rtol=1e-13, atol=1e-14)
    assert np.allclose(ATY, A.T @ Y, rtol=1e-13, atol=1e-14)
    assert not np.allclose(AX, A.T @ X, rtol=1e-6)
    assert math.isclose(np.sum(AX * Y), np.sum(X * ATY), rel_tol=1e-12)   # <AX,Y> = <X,A^T Y>


def test_spmm_rectangular_rows_csr():
    m, k, d = 17, 29, 6
    dense = (rng.random((m, k)) < 0.2) * rng.random((m, k))
    dense = dense.astype(np.float32)
    rowptr = np.zeros(m + 1, np.int64); cols = []; vals = []
    for i in range(m):
        nz = np.nonzero(dense[i])[0]
        cols += nz.tolist(); vals += dense[i, nz].tolist(); rowptr[i + 1] = len(cols)
    cols = np.array(cols, np.int32); vals = np.array(vals, np.float32)
    X = rng.standard_normal((k, d)).astype(np.float32)
    G = rng.standard_normal((m, d)).astype(np.float32)
    sample = np.array([0, 5, 16, 5])
    out = oracle.spmm_rows_csr(rowptr, cols, vals, X, sample)
    assert np.allclose(out, (dense.astype(np.float64) @ X.astype(np.float64))[sample], rtol=1e-13)
    sample_t = np.array([28, 0, 7, 7, 13])
    out_t = oracle.spmm_t_rows_csr(m, k, rowptr, cols, vals, G, sample_t)
    assert np.allclose(out_t, (dense.astype(np.float64).T @ G.astype(np.float64))[sample_t], rtol=1e-13)


@pytest.mark.parametrize("ta,tb", [(False, False), (True, False), (False, True), (True, True)])
def test_gemm_against_numpy(ta, tb):
    M, N, K = 7, 5, 11
    A = rng.standard_normal((K, M) if ta else (M, K))
    B = rng.standard_normal((N, K) if tb else (K, N))
    ref = (A.T if ta else A) @ (B.T if tb else B)
    assert np.allclose(oracle.gemm(A, B, ta, tb), ref, rtol=1e-13, atol=1e-14)
    I = np.eye(K)
    if not ta and not tb:
        assert np.array_equal(oracle.gemm(A, I), A)


def test_relu_and_softmax_closed_forms():
    z = np.array([[-1.0, 0.0, 2.5]])
    assert np.array_equal(oracle.relu(z), [[0.0, 0.0, 2.5]])
    assert np.array_equal(oracle.relu_bwd(z, np.ones_like(z)), [[0.0, 0.0, 1.0]])   # ReLU'(0) = 0
    # uniform logits: loss = log C, gradient = (1/C - onehot)/n
    n, c = 4, 5
    loss, dZ = oracle.softmax_ce(np.zeros((n, c)), np.array([0, 1, 2, 3]))
    assert math.isclose(loss, math.log(c), rel_tol=1e-15)
    assert math.isclose(dZ[0, 0], (1 / c - 1) / n) and math.isclose(dZ[0, 1], 1 / c / n)
    assert np.allclose(dZ.sum(axis=1), 0.0, atol=1e-16)
    # a confidently right prediction has ~zero loss; shift invariance
    Z = rng.standard_normal((n, c))
    l1, _ = oracle.softmax_ce(Z, np.array([0, 1, 2, 3]))
    l2, _ = oracle.softmax_ce(Z + 100.0, np.array([0, 1, 2, 3]))
    assert math.isclose(l1, l2, rel_tol=1e-12)
    big = np.full((1, 3), -50.0); big[0, 1] = 50.0
    assert oracle.softmax_ce(big, np.array([1]))[0] < 1e-40


# ---------------------------------------------------------------- whole network

def tiny_problem(n=36, e=110, dims=(6, 5, 4, 3), seed=5):
    n, src, dst = small_graph(n, e, seed)
    r = np.random.default_rng(seed + 1)
    F0 = r.standard_normal((n, dims[0]))
    Ws = [r.standard_normal((dims[i], dims[i + 1])) * 0.7 for i in range(len(dims) - 1)]
    y = r.integers(0, dims[-1], n)
    return n, src, dst, F0, Ws, y


def test_network_matches_dense_brute_force():
    n, src, dst, F0, Ws, y = tiny_problem()
    adj = oracle.adjacency(n, src, dst)
    t = ogcn.forward_backward(adj, F0, Ws, y)
    A, _ = odense.dense_adjacency(n, src, dst)
    Z, loss, dWs, dF0 = odense.gcn_forward_backward(A, F0, Ws, y)
    assert np.allclose(t.logits, Z, rtol=1e-12, atol=1e-13)
    assert math.isclose(t.loss, loss, rel_tol=1e-12)
    for a, b in zip(t.dW, dWs):
        assert np.allclose(a, b, rtol=1e-11, atol=1e-14)
    assert np.allclose(t.dF[0], dF0, rtol=1e-11, atol=1e-15)


def test_empty_graph_reduces_to_plain_gemm():
    n, _, _, F0, Ws, y = tiny_problem()
    adj = oracle.adjacency(n, np.zeros(0, np.int64), np.zeros(0, np.int64))
    t = ogcn.forward(adj, F0, Ws[:1])
    assert np.allclose(t.logits, F0 @ Ws[0], rtol=1e-14)


def test_complete_graph_gives_column_means():
    n = 12
    iu = np.triu_indices(n, 1)
    adj = oracle.adjacency(n, iu[0], iu[1])
    F0 = rng.standard_normal((n, 4)); W = rng.standard_normal((4, 3))
    t = ogcn.forward(adj, F0, [W])
    assert np.allclose(t.logits, np.tile((F0 @ W).mean(axis=0), (n, 1)), rtol=1e-13)


def test_finite_difference_gradients():
    """Central differences of the fp64 loss against dW of every layer and dF0 (Eq. 2.4-2.7)."""
    n, src, dst, F0, Ws, y = tiny_problem(n=24, e=70, dims=(4, 5, 3))
    adj = oracle.adjacency(n, src, dst)
    t = ogcn.forward_backward(adj, F0, Ws, y)
    h = 1e-6
    r = np.random.default_rng(0)
    for l, W in enumerate(Ws):
        for _ in range(6):
            i, j = r.integers(0, W.shape[0]), r.integers(0, W.shape[1])
            Wp = [w.copy() for w in Ws]; Wm = [w.copy() for w in Ws]
            Wp[l][i, j] += h; Wm[l][i, j] -= h
            fd = (ogcn.loss_only(adj, F0, Wp, y) - ogcn.loss_only(adj, F0, Wm, y)) / (2 * h)
            assert math.isclose(fd, t.dW[l][i, j], rel_tol=2e-5, abs_tol=1e-9), (l, i, j)
    for _ in range(8):
        i, j = r.integers(0, n), r.integers(0, F0.shape[1])
        Fp = F0.copy(); Fm = F0.copy()
        Fp[i, j] += h; Fm[i, j] -= h
        fd = (ogcn.loss_only(adj, Fp, Ws, y) - ogcn.loss_only(adj, Fm, Ws, y)) / (2 * h)
        assert math.isclose(fd, t.dF[0][i, j], rel_tol=2e-5, abs_tol=1e-9), (i, j)


# ---------------------------------------------------------------- permutations (Sec. 5.1)

def test_permuted_csr_against_permutation_matrices():
    """P_r A^ P_c^T built from explicit permutation matrices equals the canonical CSR, and
    the transposed orientation P_c A^ P_r^T is its transpose (A^ symmetric)."""
    n, src, dst = small_graph(30, 90, 21)
    adj = oracle.adjacency(n, src, dst)
    A = to_dense(adj)
    r = np.random.default_rng(2)
    pr, pc = r.permutation(n), r.permutation(n)
    Pr, Pc = odense.permutation_matrix(pr), odense.permutation_matrix(pc)
    rowptr, col, val = oracle.permuted_csr(adj, pr, pc)
    B = np.zeros((n, n), np.float32)
    for i in range(n):
        cs = col[rowptr[i]:rowptr[i + 1]]
        assert np.all(np.diff(cs) > 0)                            # strictly ascending columns
        B[i, cs] = val[rowptr[i]:rowptr[i + 1]]
    assert np.array_equal(B, (Pr @ A @ Pc.T).astype(np.float32))
    rowptr2, col2, val2 = oracle.permuted_csr(adj, pc, pr)
    B2 = np.zeros((n, n), np.float32)
    for i in range(n):
        B2[i, col2[rowptr2[i]:rowptr2[i + 1]]] = val2[rowptr2[i]:rowptr2[i + 1]]
    assert np.array_equal(B2, B.T)
    with pytest.raises(ValueError):
        bad = pr.copy(); bad[0] = bad[1]
        oracle.permuted_csr(adj, bad, pc)


def test_double_permutation_invariance_of_the_network():
    """Eq. 5.3-5.4: running the layers on P_r A P_c^T / P_c A P_r^T alternately, with input
    P_c F0, gives the unpermuted network's output up to the row relabelling."""
    n, src, dst, F0, Ws, y = tiny_problem(n=40, e=140, dims=(5, 6, 4, 3))
    adj = oracle.adjacency(n, src, dst)
    ref = ogcn.forward(adj, F0, Ws)
    A = to_dense(adj)
    r = np.random.default_rng(9)
    pr, pc = r.permutation(n), r.permutation(n)
    Pr, Pc = odense.permutation_matrix(pr), odense.permutation_matrix(pc)
    A_even, A_odd = Pr @ A @ Pc.T, Pc @ A @ Pr.T
    F = Pc @ F0
    for l, W in enumerate(Ws):
        Q = (A_even if l % 2 == 0 else A_odd) @ F @ W
        F = np.maximum(Q, 0.0)
    out_perm = pr if (len(Ws) - 1) % 2 == 0 else pc               # last layer even -> P_r order
    assert np.allclose(Q[out_perm], ref.logits, rtol=1e-12, atol=1e-13)
    # single permutation, Eq. 5.1-5.2
    As = Pr @ A @ Pr.T
    F = Pr @ F0
    for W in Ws:
        Q = As @ F @ W
        F = np.maximum(Q, 0.0)
    assert np.allclose(Q[pr], ref.logits, rtol=1e-12, atol=1e-13)


def test_block_balance_table3():
    """Table 3: single permutation keeps all N self-loops in the diagonal blocks, so
    max/mean = (nnz_off/B^2 + N/B) / (nnz/B^2); with Table 4's europe_osm row this is the
    printed 3.24.  The same closed form is then checked on a synthetic road-like graph, and
    the double permutation brings the ratio close to 1 as the table says."""
    t4 = {r[0]: list(map(int, r[1:])) for r in read_table("table4_datasets.txt")}
    t3 = {r[0]: float(r[1]) for r in read_table("table3_balance.txt")}
    N, _, nnz = t4["europe_osm"][:3]
    B = 8
    closed = ((nnz - N) / B**2 + N / B) / (nnz / B**2)
    assert abs(closed - t3["single_permutation"]) < 0.005
    cfg = synth.CONFIGS["road"].scaled(4e-3)
    src, dst = cfg.edges()
    adj = oracle.adjacency(cfg.n, src.numpy(), dst.numpy())
    pr, pc = (p.numpy() for p in cfg.perms())
    orig = odense.block_balance(cfg.n, adj.row, adj.col, B)
    single = odense.block_balance(cfg.n, pr[adj.row], pr[adj.col], B)
    double = odense.block_balance(cfg.n, pr[adj.row], pc[adj.col], B)
    expect_single = ((adj.nnz - cfg.n) / B**2 + cfg.n / B) / (adj.nnz / B**2)
    assert orig > single > double
    assert abs(single - expect_single) / expect_single < 0.02
    assert double < 1.03
    assert abs(t3["double_permutation"] - 1.0) < 0.01


def test_sampled_rows_against_dense_brute_force():
    """oracle.sampled (single rows from the definition, used at full size) against the dense
    P_r A^ P_c^T built from permutation matrices."""
    from oracle import sampled as osampled
    n = 37
    r = np.random.default_rng(4)
    pairs = {(min(u, v), max(u, v)) for u, v in zip(r.integers(0, n, 120).tolist(), r.integers(0, n, 120).tolist()) if u != v}
    src = np.array([p[0] for p in pairs]); dst = np.array([p[1] for p in pairs])      # distinct, loop-free
    A, d = odense.dense_adjacency(n, src, dst)
    pr, pc = r.permutation(n), r.permutation(n)
    B = (odense.permutation_matrix(pr) @ A @ odense.permutation_matrix(pc).T).astype(np.float32)
    deg = osampled.degrees(n, src, dst)
    assert np.array_equal(deg, d)
    rows = osampled.permuted_rows(n, src, dst, deg, pr, pc, np.arange(n))
    assert sorted(rows) == list(range(n))
    for i, (cols, vals) in rows.items():
        assert np.all(np.diff(cols) > 0)
        dense_row = np.zeros(n, np.float32); dense_row[cols] = vals
        assert np.array_equal(dense_row, B[i])


def distinct_edges(n, e, seed):
    r = np.random.default_rng(seed)
    pairs = {(min(u, v), max(u, v)) for u, v in zip(r.integers(0, n, e).tolist(), r.integers(0, n, e).tolist()) if u != v}
    return np.array([p[0] for p in pairs]), np.array([p[1] for p in pairs])


def test_sampled_adjacency_rows_against_dense_brute_force():
    from oracle import sampled as osampled
    n = 41
    src, dst = distinct_edges(n, 90, 8)
    A, d = odense.dense_adjacency(n, src, dst)
    rows = osampled.adjacency_rows(n, src, dst, osampled.degrees(n, src, dst), np.array([0, 5, 17, 40]))
    for u, (ids, vals) in rows.items():
        dense_row = np.zeros(n); dense_row[ids] = vals
        assert np.array_equal(ids, np.nonzero(A[u])[0])
        assert np.allclose(dense_row, A[u], rtol=1e-15, atol=0)


@pytest.mark.parametrize("dims", [(5, 6, 3), (4, 7, 5, 3)])
def test_network_on_samples_equals_the_whole_graph_network(dims):
    """oracle.sampled.network_on_samples (the network evaluated on the receptive field of a few nodes, used at
    full size) against the dense brute force on the whole graph with the same loss gradient: logits on the
    samples, dW of every layer, dF0 on the field, zero dF0 outside it."""
    from oracle import sampled as osampled
    n = 60
    src, dst = distinct_edges(n, 55, 3)                       # sparse: the field of 4 nodes is not the whole graph
    r = np.random.default_rng(11)
    F0 = r.standard_normal((n, dims[0]))
    Ws = [r.standard_normal((dims[l], dims[l + 1])) * 0.5 for l in range(len(dims) - 1)]
    nodes = np.array([3, 31, 32, 58])
    g = r.standard_normal((len(nodes), dims[-1]))
    V, logits, dW, dF0, Q = osampled.network_on_samples(n, src, dst, osampled.degrees(n, src, dst), lambda ids: F0[ids], Ws, nodes, g)
    assert len(V[-1]) < n
    # the whole graph, dense numpy: forward, then Eq. 2.4-2.7 from the same gradient
    A, _ = odense.dense_adjacency(n, src, dst)
    F, Hs, Qs = F0, [], []
    for l, W in enumerate(Ws):
        Hs.append(A @ F); Qs.append(Hs[l] @ W)
        F = np.maximum(Qs[l], 0.0)
    dQ = np.zeros((n, dims[-1])); dQ[nodes] = g
    for l in range(len(Ws) - 1, -1, -1):
        if l + 1 < len(Ws):
            dQ = dF * (Qs[l] > 0)
        assert np.allclose(dW[l], Hs[l].T @ dQ, rtol=1e-11, atol=1e-13), l
        dF = A.T @ (dQ @ Ws[l].T)
    assert np.allclose(logits, Qs[-1][nodes], rtol=1e-12, atol=1e-13)
    assert np.allclose(dF0, dF[V[-1]], rtol=1e-11, atol=1e-14)
    outside = np.setdiff1d(np.arange(n), V[-1])
    assert np.all(dF[outside] == 0.0)
    assert np.allclose(Q[0], Qs[0][V[len(Ws) - 1]], rtol=1e-12, atol=1e-13)


def test_backward_with_given_masks():
    """masks = [Q > 0] reproduces the plain backward pass; a flipped entry changes exactly what a finite difference of
    the correspondingly modified activation function gives (here: checked through the dense form)."""
    n, src, dst, F0, Ws, y = tiny_problem()
    adj = oracle.adjacency(n, src, dst)
    t = ogcn.forward_backward(adj, F0, Ws, y)
    masks = [(q > 0) for q in t.Q[:-1]] + [None]
    t2 = ogcn.forward_backward(adj, F0, Ws, y, masks=masks)
    for a, b in zip(t.dW + [t.dF[0]], t2.dW + [t2.dF[0]]):
        assert np.array_equal(a, b)
    flipped = [m.copy() for m in masks[:-1]] + [None]
    flipped[0][2, 1] = ~flipped[0][2, 1]
    t3 = ogcn.forward_backward(adj, F0, Ws, y, masks=flipped)
    A, _ = odense.dense_adjacency(n, src, dst)
    # dense reference with the same decisions
    F, Hs, Qs = F0, [], []
    for l, W in enumerate(Ws):
        Hs.append(A @ F); Qs.append(Hs[l] @ W); F = np.maximum(Qs[l], 0.0)
    e = np.exp(Qs[-1] - Qs[-1].max(axis=1, keepdims=True)); p = e / e.sum(axis=1, keepdims=True)
    dQ = p.copy(); dQ[np.arange(n), y] -= 1.0; dQ /= n
    for l in range(len(Ws) - 1, -1, -1):
        if l + 1 < len(Ws):
            dQ = dF * flipped[l]
        assert np.allclose(t3.dW[l], Hs[l].T @ dQ, rtol=1e-11, atol=1e-14)
        dF = A.T @ (dQ @ Ws[l].T)
    assert not np.allclose(t3.dW[0], t.dW[0], rtol=1e-9, atol=0)
