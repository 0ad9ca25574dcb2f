"""CPU oracle for the GCN hot path -- TEST INFRASTRUCTURE, not part of the product.

Only `tests/`, `__graft_entry__.smoke()` and `bench.py`'s cpu_baseline leg may import this
package.  It shares no code with the HIP library and never imports it.

Two independent forms of the same mathematics:

* `oracle.plx_oracle.c` (bound here through ctypes): coordinate-list loops in fp64, following
  Sec. 2.1 (normalised adjacency with self-loops), Eq. 2.1-2.7 (layer forward / backward) and
  Eq. 5.3-5.4 (double permutation) of the paper.
* `oracle.dense`: a dense N x N brute force in numpy for tiny graphs.

`oracle.gcn` composes the C steps into an L-layer forward + backward on the UNPERMUTED graph.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "plx_oracle.c")
# PLX_ORACLE_SANITIZE=1: an AddressSanitizer + UndefinedBehaviorSanitizer build of the same source, kept beside the
# plain one (the process must then run with the ASan runtime preloaded; tests/test_oracle_sanitized.py does that)
_SANITIZE = os.environ.get("PLX_ORACLE_SANITIZE", "") == "1"
_SO = os.path.join(_HERE, "libplx_oracle_san.so" if _SANITIZE else "libplx_oracle.so")

_i64p = ctypes.POINTER(ctypes.c_int64)
_i32p = ctypes.POINTER(ctypes.c_int32)
_f64p = ctypes.POINTER(ctypes.c_double)
_f32p = ctypes.POINTER(ctypes.c_float)
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math: fp64 sqrt/div stay correctly rounded)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-ffp-contract=off",
               "-fvisibility=hidden", "-o", _SO, _SRC, "-lm"]
        if _SANITIZE:
            cmd[1:2] = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
        subprocess.check_call(cmd)
    return _SO


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_SO)
        L.orc_num_threads.restype = ctypes.c_int
        L.orc_set_num_threads.argtypes = [ctypes.c_int]
        L.orc_adj_build.restype = ctypes.c_int64
        L.orc_adj_build.argtypes = [ctypes.c_int64, ctypes.c_int64, _i64p, _i64p, _i64p, _i64p, _f64p, _i64p]
        L.orc_permuted_csr.restype = ctypes.c_int
        L.orc_permuted_csr.argtypes = [ctypes.c_int64, ctypes.c_int64, _i64p, _i64p, _i64p, _i64p, _i64p,
                                       _i64p, _i32p, _f32p]
        L.orc_spmm_coo.restype = None
        L.orc_spmm_coo.argtypes = [ctypes.c_int64, ctypes.c_int64, _i64p, _i64p, _f64p, _f64p, ctypes.c_int64,
                                   _f64p, ctypes.c_int64, ctypes.c_int64]
        L.orc_spmm_t_coo.restype = None
        L.orc_spmm_t_coo.argtypes = L.orc_spmm_coo.argtypes
        L.orc_spmm_rows_csr.restype = None
        L.orc_spmm_rows_csr.argtypes = [_i64p, _i32p, _f32p, _f32p, ctypes.c_int64, ctypes.c_int64,
                                        _i64p, ctypes.c_int64, _f64p]
        L.orc_spmm_t_rows_csr.restype = None
        L.orc_spmm_t_rows_csr.argtypes = [ctypes.c_int64, ctypes.c_int64, _i64p, _i32p, _f32p, _f64p,
                                          ctypes.c_int64, ctypes.c_int64, _i64p, ctypes.c_int64, _f64p]
        L.orc_gemm.restype = None
        L.orc_gemm.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                               _f64p, ctypes.c_int64, _f64p, ctypes.c_int64, _f64p, ctypes.c_int64]
        L.orc_relu.restype = None
        L.orc_relu.argtypes = [ctypes.c_int64, _f64p, _f64p]
        L.orc_relu_bwd.restype = None
        L.orc_relu_bwd.argtypes = [ctypes.c_int64, _f64p, _f64p, _f64p]
        L.orc_softmax_ce.restype = ctypes.c_double
        L.orc_softmax_ce.argtypes = [ctypes.c_int64, ctypes.c_int64, _f64p, ctypes.c_int64, _i64p, _f64p,
                                     ctypes.c_int64]
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray], typ):
    return None if a is None else a.ctypes.data_as(typ)


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=dtype)


def num_threads() -> int:
    return int(lib().orc_num_threads())


def set_num_threads(t: int) -> None:
    lib().orc_set_num_threads(int(t))


class Adjacency:
    """Normalised adjacency with self-loops (Sec. 2.1) as a coordinate list in original ids."""

    def __init__(self, n, row, col, val, deg):
        self.n, self.row, self.col, self.val, self.deg = n, row, col, val, deg

    @property
    def nnz(self) -> int:
        return int(self.row.shape[0])


def adjacency(n: int, src, dst) -> Adjacency:
    src, dst = _c(src, np.int64), _c(dst, np.int64)
    ne = src.shape[0]
    cap = 2 * ne + n
    row = np.empty(cap, np.int64); col = np.empty(cap, np.int64); val = np.empty(cap, np.float64)
    deg = np.empty(max(n, 1), np.int64)
    nnz = lib().orc_adj_build(n, ne, _p(src, _i64p), _p(dst, _i64p), _p(row, _i64p), _p(col, _i64p),
                              _p(val, _f64p), _p(deg, _i64p))
    if nnz < 0:
        raise ValueError("edge list holds a node id outside [0, n)")
    return Adjacency(n, row[:nnz].copy(), col[:nnz].copy(), val[:nnz].copy(), deg[:n].copy())


def permuted_csr(adj: Adjacency, perm_r=None, perm_c=None) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(rowptr int64[n+1], col int32[nnz], val float32[nnz]) of P_r A^ P_c^T (Eq. 5.3)."""
    pr = None if perm_r is None else _c(perm_r, np.int64)
    pc = None if perm_c is None else _c(perm_c, np.int64)
    rowptr = np.empty(adj.n + 1, np.int64); col = np.empty(max(adj.nnz, 1), np.int32)
    val = np.empty(max(adj.nnz, 1), np.float32)
    rc = lib().orc_permuted_csr(adj.n, adj.nnz, _p(adj.row, _i64p), _p(adj.col, _i64p), _p(adj.deg, _i64p),
                                _p(pr, _i64p), _p(pc, _i64p), _p(rowptr, _i64p), _p(col, _i32p), _p(val, _f32p))
    if rc != 0:
        raise ValueError("permutation is not a bijection on [0, n)")
    return rowptr, col[:adj.nnz], val[:adj.nnz]


def spmm_coo(m: int, row, col, val, X) -> np.ndarray:
    """Y = A X (Eq. 2.1); `row` ascending."""
    row, col, val = _c(row, np.int64), _c(col, np.int64), _c(val, np.float64)
    X = _c(X, np.float64)
    d = X.shape[1]
    Y = np.empty((m, d), np.float64)
    lib().orc_spmm_coo(m, row.shape[0], _p(row, _i64p), _p(col, _i64p), _p(val, _f64p), _p(X, _f64p), d,
                       _p(Y, _f64p), d, d)
    return Y


def spmm_t_coo(k: int, row, col, val, X) -> np.ndarray:
    """Y = A^T X (Eq. 2.7)."""
    row, col, val = _c(row, np.int64), _c(col, np.int64), _c(val, np.float64)
    X = _c(X, np.float64)
    d = X.shape[1]
    Y = np.empty((k, d), np.float64)
    lib().orc_spmm_t_coo(k, row.shape[0], _p(row, _i64p), _p(col, _i64p), _p(val, _f64p), _p(X, _f64p), d,
                         _p(Y, _f64p), d, d)
    return Y


def spmm_rows_csr(rowptr, col, val, X, sample) -> np.ndarray:
    """Rows `sample` of A X for a CSR block with fp32 values and an fp32 operand."""
    rowptr, col, val = _c(rowptr, np.int64), _c(col, np.int32), _c(val, np.float32)
    X, sample = _c(X, np.float32), _c(sample, np.int64)
    d = X.shape[1]
    out = np.empty((sample.shape[0], d), np.float64)
    lib().orc_spmm_rows_csr(_p(rowptr, _i64p), _p(col, _i32p), _p(val, _f32p), _p(X, _f32p), d, d,
                            _p(sample, _i64p), sample.shape[0], _p(out, _f64p))
    return out


def spmm_t_rows_csr(m: int, k: int, rowptr, col, val, X, sample) -> np.ndarray:
    """Rows `sample` of A^T X for the same kind of block (X is widened to fp64)."""
    rowptr, col, val = _c(rowptr, np.int64), _c(col, np.int32), _c(val, np.float32)
    X, sample = _c(X, np.float64), _c(sample, np.int64)
    d = X.shape[1]
    out = np.empty((sample.shape[0], d), np.float64)
    lib().orc_spmm_t_rows_csr(m, k, _p(rowptr, _i64p), _p(col, _i32p), _p(val, _f32p), _p(X, _f64p), d, d,
                              _p(sample, _i64p), sample.shape[0], _p(out, _f64p))
    return out


def gemm(A, B, ta: bool = False, tb: bool = False) -> np.ndarray:
    """op(A) op(B) by the triple loop (Eq. 2.2, 2.5, 2.6)."""
    A, B = _c(A, np.float64), _c(B, np.float64)
    M = A.shape[1] if ta else A.shape[0]
    K = A.shape[0] if ta else A.shape[1]
    Kb = B.shape[1] if tb else B.shape[0]
    N = B.shape[0] if tb else B.shape[1]
    if K != Kb:
        raise ValueError("inner dimensions differ")
    C = np.empty((M, N), np.float64)
    lib().orc_gemm(int(ta), int(tb), M, N, K, _p(A, _f64p), A.shape[1], _p(B, _f64p), B.shape[1], _p(C, _f64p), N)
    return C


def relu(Z) -> np.ndarray:
    Z = _c(Z, np.float64)
    F = np.empty_like(Z)
    lib().orc_relu(Z.size, _p(Z, _f64p), _p(F, _f64p))
    return F


def relu_bwd(Z, dF) -> np.ndarray:
    Z, dF = _c(Z, np.float64), _c(dF, np.float64)
    dZ = np.empty_like(Z)
    lib().orc_relu_bwd(Z.size, _p(Z, _f64p), _p(dF, _f64p), _p(dZ, _f64p))
    return dZ


def softmax_ce(Z, y) -> Tuple[float, np.ndarray]:
    """(mean cross-entropy, dZ = (softmax - onehot)/n)."""
    Z, y = _c(Z, np.float64), _c(y, np.int64)
    n, c = Z.shape
    dZ = np.empty_like(Z)
    loss = lib().orc_softmax_ce(n, c, _p(Z, _f64p), c, _p(y, _i64p), _p(dZ, _f64p), c)
    return float(loss), dZ
