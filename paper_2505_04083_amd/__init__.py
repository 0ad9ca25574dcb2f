"""Thin Python binding of the plx C ABI (include/plx.h): argument marshalling only.

Every function here has the name of the C entry point it calls and takes torch tensors where
the C function takes device pointers.  torch supplies device memory and the HIP stream; all
arithmetic runs in the library's own kernels.  There is no fallback: if the shared library
cannot be loaded the import fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libplx.so")

PLX_OK, PLX_ERR_INVALID, PLX_ERR_SHAPE, PLX_ERR_UNSUPPORTED, PLX_ERR_OOM, PLX_ERR_DEVICE, PLX_ERR_INTERNAL = range(7)
PLX_F32, PLX_BF16 = 0, 1
PLX_ACT_NONE, PLX_ACT_RELU, PLX_ACT_RELU_BITS = 0, 1, 2
PLX_ORDER_COMBINE_FIRST, PLX_ORDER_AGG_FIRST, PLX_ORDER_AUTO = 0, 1, 2

EXPORTED = [
    "plx_ctx_create", "plx_ctx_destroy", "plx_ctx_set_column_windows", "plx_ctx_set_split_products", "plx_ctx_set_fused_aggregation", "plx_last_error", "plx_status_string", "plx_sync",
    "plx_timing_enable", "plx_timing_report", "plx_timing_trace",
    "plx_build_csr", "plx_csr_import", "plx_csr_dims", "plx_csr_export", "plx_csr_bins", "plx_csr_destroy",
    "plx_csr_set_row_blocks", "plx_csr_row_blocks", "plx_spmm_block", "plx_spmm", "plx_spmm_t", "plx_spmm_static", "plx_gemm_nn", "plx_gemm_nt", "plx_gemm_tn_workspace", "plx_gemm_tn",
    "plx_relu", "plx_relu_bwd", "plx_softmax_ce",
    "plx_gcn_layer_workspace", "plx_gcn_layer_fwd", "plx_gcn_layer_bwd",
    "plx_gcn_layer_bwd_dt", "plx_gcn_layer_bwd_chained_workspace", "plx_gcn_layer_bwd_chained",
    "plx_gcn_layer_fwd_chained", "plx_gcn_layer_fwd_from_t", "plx_gcn_layer_plan",
]

_ALLOC_FN = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p)
_FREE_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_void_p)

_vp, _i64, _int, _sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t


def _load() -> ctypes.CDLL:
    if not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build(verbose=False)
    lib = ctypes.CDLL(_LIB_PATH)
    sig = {
        "plx_ctx_create": (_int, [_int, _vp, _ALLOC_FN, _FREE_FN, _vp, ctypes.POINTER(_vp)]),
        "plx_ctx_destroy": (None, [_vp]),
        "plx_last_error": (ctypes.c_char_p, [_vp]),
        "plx_status_string": (ctypes.c_char_p, [_int]),
        "plx_sync": (_int, [_vp]),
        "plx_timing_enable": (_int, [_vp, _int]),
        "plx_timing_report": (_int, [_vp, ctypes.c_char_p, _sz]),
        "plx_timing_trace": (_int, [_vp, ctypes.c_char_p, _sz]),
        "plx_build_csr": (_int, [_vp, _i64, _i64, _vp, _vp, _vp, _vp, ctypes.POINTER(_vp)]),
        "plx_csr_import": (_int, [_vp, _i64, _i64, _i64, _vp, _vp, _vp, ctypes.POINTER(_vp)]),
        "plx_csr_dims": (_int, [_vp, ctypes.POINTER(_i64), ctypes.POINTER(_i64), ctypes.POINTER(_i64)]),
        "plx_csr_export": (_int, [_vp, _vp, _int, _vp, _vp, _vp, _vp]),
        "plx_csr_bins": (_int, [_vp, _int, ctypes.POINTER(_i64), ctypes.POINTER(_i64)]),
        "plx_csr_destroy": (None, [_vp, _vp]),
        "plx_ctx_set_column_windows": (_int, [_vp, _int]),
        "plx_ctx_set_split_products": (_int, [_vp, _int]),
        "plx_ctx_set_fused_aggregation": (_int, [_vp, _int]),
        "plx_csr_set_row_blocks": (_int, [_vp, _vp, _int]),
        "plx_csr_row_blocks": (_int, [_vp, _int, ctypes.POINTER(_int), ctypes.POINTER(_i64)]),
        "plx_spmm_block": (_int, [_vp, _vp, _int, _int, _vp, _i64, _vp, _i64, _i64, _int]),
        "plx_spmm": (_int, [_vp, _vp, _vp, _i64, _vp, _i64, _i64, _int]),
        "plx_spmm_static": (_int, [_vp, _vp, _int, _vp, _i64, _vp, _i64, _i64, _int]),
        "plx_spmm_t": (_int, [_vp, _vp, _vp, _i64, _vp, _i64, _i64, _int]),
        "plx_gemm_nn": (_int, [_vp, _i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _int]),
        "plx_gemm_nt": (_int, [_vp, _i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _int]),
        "plx_gemm_tn_workspace": (_sz, [_i64, _i64, _i64]),
        "plx_gemm_tn": (_int, [_vp, _i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _int, _vp, _sz]),
        "plx_relu": (_int, [_vp, _i64, _i64, _vp, _i64, _vp, _i64, _int]),
        "plx_relu_bwd": (_int, [_vp, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _int]),
        "plx_softmax_ce": (_int, [_vp, _i64, _i64, _vp, _i64, _vp, _vp, _i64, _vp, _vp, _int]),
        "plx_gcn_layer_workspace": (_sz, [_vp, _int, _i64, _i64, _int, _int, _int]),
        "plx_gcn_layer_fwd": (_int, [_vp, _vp, _int, _vp, _i64, _vp, _i64, _i64, _i64, _int, _int, _int,
                                     _vp, _i64, _vp, _i64, _vp, _i64, _vp, _sz]),
        "plx_gcn_layer_bwd": (_int, [_vp, _vp, _int, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64,
                                     _i64, _i64, _int, _int, _int, _vp, _i64, _vp, _i64, _vp, _sz]),
        "plx_gcn_layer_fwd_chained": (_int, [_vp, _vp, _int, _vp, _i64, _vp, _i64, _i64, _i64, _int, _int, _int,
                                             _vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _i64, _vp, _i64, _vp, _sz]),
        "plx_gcn_layer_fwd_from_t": (_int, [_vp, _vp, _int, _vp, _i64, _i64, _int, _int, _vp, _i64, _vp, _i64]),
        "plx_gcn_layer_bwd_dt": (_int, [_vp, _vp, _int, _vp, _i64, _vp, _i64, _vp, _i64, _i64, _i64, _int, _int,
                                        _vp, _i64, _vp, _i64, _vp, _sz]),
        "plx_gcn_layer_plan": (_int, [_vp, _i64, _i64, _i64, _int, _int, _int, _int, ctypes.POINTER(_int), ctypes.POINTER(_int),
                                      ctypes.POINTER(_int), ctypes.POINTER(_int)]),
        "plx_gcn_layer_bwd_chained_workspace": (_sz, [_vp, _vp, _int, _i64, _i64, _i64, _int, _int, _int]),
        "plx_gcn_layer_bwd_chained": (_int, [_vp, _vp, _int, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _i64,
                                             _vp, _i64, _i64, _i64, _int, _int, _int, _vp, _i64, _vp, _i64, _vp, _sz]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)          # AttributeError if the library lacks a declared symbol
        fn.restype = res
        fn.argtypes = args
    return lib


_lib = _load()


class PlxError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"plx status {status} ({_lib.plx_status_string(status).decode()}): {message}")
        self.status = status


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return PLX_F32
    if t.dtype == torch.bfloat16:
        return PLX_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _mat(t: Optional[torch.Tensor]) -> Tuple[Optional[int], int]:
    """(pointer, leading dimension in elements) of a row-major 2-D tensor."""
    if t is None:
        return None, 0
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("expected a row-major 2-D tensor")
    ld = t.stride(0) if t.shape[0] > 1 else max(t.shape[1], t.stride(0))
    return t.data_ptr(), int(ld)


def _check(ctx: "plx_ctx", name: str, t: Optional[torch.Tensor], rows: int, cols: int, dtype=None) -> None:
    """The C ABI sees pointers and leading dimensions only: that the memory behind them is on the context's GPU, of
    the element type the call says and large enough is checked here, before the call (ValueError / TypeError)."""
    if t is None:
        return
    if ctx.device >= 0 and (not t.is_cuda or t.device.index != ctx.device):
        raise ValueError(f"{name}: tensor on {t.device}, the context runs on cuda:{ctx.device}")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if t.dim() != 2 or t.shape[0] < rows or t.shape[1] < cols:
        raise ValueError(f"{name}: shape {tuple(t.shape)} smaller than the {rows} x {cols} the call addresses")


def _check_ws(ctx: "plx_ctx", ws: Optional[torch.Tensor]) -> None:
    if ws is None:
        return
    if ctx.device >= 0 and (not ws.is_cuda or ws.device.index != ctx.device):
        raise ValueError(f"workspace on {ws.device}, the context runs on cuda:{ctx.device}")
    if ws.dtype != torch.uint8 or not ws.is_contiguous():
        raise TypeError("the workspace is a contiguous uint8 tensor")


def _ptr(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError("expected a contiguous tensor")
    return t.data_ptr()


class plx_ctx:
    """A library context bound to one GPU and one HIP stream (torch's current stream by
    default).  device=-1 makes a validate-only context (no GPU needed).  With
    torch_allocator=True the library's own buffers come from torch's caching allocator."""

    def __init__(self, device: Optional[int] = None, stream: Optional[int] = None, torch_allocator: bool = True):
        if device is None:
            device = torch.cuda.current_device()
        self.device = device
        self._live = {}
        self.handle = _vp()
        if device >= 0 and torch_allocator:
            dev = torch.device("cuda", device)

            def _alloc(nbytes, _user):
                try:
                    t = torch.empty(int(nbytes), dtype=torch.uint8, device=dev)
                except Exception:
                    return None
                self._live[t.data_ptr()] = t
                return t.data_ptr()

            def _free(p, _user):
                self._live.pop(p, None)

            self._alloc_cb, self._free_cb = _ALLOC_FN(_alloc), _FREE_FN(_free)
        else:
            self._alloc_cb, self._free_cb = _ALLOC_FN(0), _FREE_FN(0)
        if stream is None and device >= 0:
            stream = torch.cuda.current_stream(device).cuda_stream
        st = _lib.plx_ctx_create(device, stream, self._alloc_cb, self._free_cb, None, ctypes.byref(self.handle))
        if st != PLX_OK:
            raise PlxError(st, "plx_ctx_create failed")

    def check(self, status: int) -> None:
        if status != PLX_OK:
            raise PlxError(status, _lib.plx_last_error(self.handle).decode())

    def close(self) -> None:
        if self.handle:
            _lib.plx_ctx_destroy(self.handle)
            self.handle = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class plx_csr:
    """Handle of a stored adjacency (both orientations)."""

    def __init__(self, ctx: plx_ctx, handle):
        self.ctx, self.handle = ctx, handle
        m, k, nnz = _i64(), _i64(), _i64()
        _lib.plx_csr_dims(handle, ctypes.byref(m), ctypes.byref(k), ctypes.byref(nnz))
        self.m, self.k, self.nnz = m.value, k.value, nnz.value

    def shape(self, transposed: bool = False) -> Tuple[int, int]:
        return (self.k, self.m) if transposed else (self.m, self.k)

    def close(self) -> None:
        if self.handle and self.ctx.handle:
            _lib.plx_csr_destroy(self.ctx.handle, self.handle)
        self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def plx_sync(ctx: plx_ctx) -> None:
    ctx.check(_lib.plx_sync(ctx.handle))


def plx_build_csr(ctx: plx_ctx, n: int, src: torch.Tensor, dst: torch.Tensor,
                  perm_r: Optional[torch.Tensor] = None, perm_c: Optional[torch.Tensor] = None) -> plx_csr:
    if src.shape != dst.shape:
        raise ValueError("src and dst differ in length")
    out = _vp()
    st = _lib.plx_build_csr(ctx.handle, n, src.numel(), _ptr(src, torch.int64), _ptr(dst, torch.int64),
                            _ptr(perm_r, torch.int64), _ptr(perm_c, torch.int64), ctypes.byref(out))
    ctx.check(st)
    return plx_csr(ctx, out)


def plx_csr_import(ctx: plx_ctx, m: int, k: int, rowptr: torch.Tensor, col: torch.Tensor, val: torch.Tensor) -> plx_csr:
    out = _vp()
    st = _lib.plx_csr_import(ctx.handle, m, k, col.numel(), _ptr(rowptr, torch.int64), _ptr(col, torch.int32),
                             _ptr(val, torch.float32), ctypes.byref(out))
    ctx.check(st)
    return plx_csr(ctx, out)


def plx_csr_export(ctx: plx_ctx, csr: plx_csr, transposed: bool = False, with_deg: bool = False):
    """(rowptr int64, col int32, val fp32[, deg int64]) as new device tensors."""
    rows = csr.k if transposed else csr.m
    dev = torch.device("cuda", ctx.device)
    rowptr = torch.empty(rows + 1, dtype=torch.int64, device=dev)
    col = torch.empty(csr.nnz, dtype=torch.int32, device=dev)
    val = torch.empty(csr.nnz, dtype=torch.float32, device=dev)
    deg = torch.empty(csr.m, dtype=torch.int64, device=dev) if with_deg else None
    ctx.check(_lib.plx_csr_export(ctx.handle, csr.handle, int(transposed), rowptr.data_ptr(), col.data_ptr(),
                                  val.data_ptr(), None if deg is None else deg.data_ptr()))
    return (rowptr, col, val, deg) if with_deg else (rowptr, col, val)


def plx_csr_bins(csr: plx_csr, transposed: bool = False):
    """((rows_subwave, rows_wave, rows_split), (entries_subwave, entries_wave, entries_split))."""
    rows, ent = (_i64 * 3)(), (_i64 * 3)()
    st = _lib.plx_csr_bins(csr.handle, int(transposed), rows, ent)
    if st != PLX_OK:
        raise PlxError(st, "plx_csr_bins")
    return tuple(rows), tuple(ent)


def plx_timing_enable(ctx: plx_ctx, on: bool) -> None:
    ctx.check(_lib.plx_timing_enable(ctx.handle, int(on)))


def plx_timing_report(ctx: plx_ctx):
    """{kernel name: (launches, total_ms)} since the last report."""
    buf = ctypes.create_string_buffer(1 << 16)
    ctx.check(_lib.plx_timing_report(ctx.handle, buf, len(buf)))
    out = {}
    for line in buf.value.decode().splitlines():
        name, count, ms = line.rsplit(" ", 2)
        out[name] = (int(count), float(ms))
    return out


def plx_timing_trace(ctx: plx_ctx, max_bytes: int = 1 << 22):
    """[(kernel name, ms)] of every timed launch since the last report, in launch order."""
    buf = ctypes.create_string_buffer(max_bytes)
    ctx.check(_lib.plx_timing_trace(ctx.handle, buf, len(buf)))
    out = []
    for line in buf.value.decode().splitlines():
        name, ms = line.rsplit(" ", 1)
        out.append((name, float(ms)))
    return out


def plx_ctx_set_split_products(ctx: plx_ctx, on: bool) -> None:
    ctx.check(_lib.plx_ctx_set_split_products(ctx.handle, int(bool(on))))


def plx_ctx_set_fused_aggregation(ctx: plx_ctx, on: bool) -> None:
    """Aggregate-first forward with the combination in the sparse kernels' epilogue (narrow fp32 layers; off by default)."""
    ctx.check(_lib.plx_ctx_set_fused_aggregation(ctx.handle, int(bool(on))))


def plx_ctx_set_column_windows(ctx: plx_ctx, n_windows: int) -> None:
    """Column windows used by handles built after this call (default 8; 1 = off)."""
    ctx.check(_lib.plx_ctx_set_column_windows(ctx.handle, n_windows))


def plx_csr_set_row_blocks(ctx: plx_ctx, csr: plx_csr, n_blocks: int) -> None:
    ctx.check(_lib.plx_csr_set_row_blocks(ctx.handle, csr.handle, n_blocks))


def plx_csr_row_blocks(csr: plx_csr, transposed: bool = False) -> Tuple[int, int]:
    """(number of row blocks, rows per block) of one orientation."""
    nb, rpb = _int(), _i64()
    st = _lib.plx_csr_row_blocks(csr.handle, int(transposed), ctypes.byref(nb), ctypes.byref(rpb))
    if st != PLX_OK:
        raise PlxError(st, "plx_csr_row_blocks")
    return nb.value, rpb.value


def plx_spmm_block(ctx: plx_ctx, csr: plx_csr, transposed: bool, block: int, X: torch.Tensor, Y: torch.Tensor,
                   d: Optional[int] = None) -> torch.Tensor:
    """Rows of row block `block` of Y = A X (or A^T X); Y is the whole output matrix."""
    xp, ldx = _mat(X)
    yp, ldy = _mat(Y)
    if d is None:
        d = X.shape[1]
    rows, cols = csr.shape(transposed)
    _check(ctx, "X", X, cols, d); _check(ctx, "Y", Y, rows, d, X.dtype)
    ctx.check(_lib.plx_spmm_block(ctx.handle, csr.handle, int(transposed), block, xp, ldx, yp, ldy, d, _dtype_code(X)))
    return Y


def _spmm(fn, ctx, csr, X, Y, d):
    xp, ldx = _mat(X)
    yp, ldy = _mat(Y)
    if d is None:
        d = X.shape[1]
    rows, cols = csr.shape(fn is _lib.plx_spmm_t)
    _check(ctx, "X", X, cols, d); _check(ctx, "Y", Y, rows, d, X.dtype)
    ctx.check(fn(ctx.handle, csr.handle, xp, ldx, yp, ldy, d, _dtype_code(X)))
    return Y


def plx_spmm(ctx: plx_ctx, csr: plx_csr, X: torch.Tensor, Y: torch.Tensor, d: Optional[int] = None) -> torch.Tensor:
    """Y[m x d] = A X[k x d]."""
    return _spmm(_lib.plx_spmm, ctx, csr, X, Y, d)


def plx_spmm_t(ctx: plx_ctx, csr: plx_csr, X: torch.Tensor, Y: torch.Tensor, d: Optional[int] = None) -> torch.Tensor:
    """Y[k x d] = A^T X[m x d]."""
    return _spmm(_lib.plx_spmm_t, ctx, csr, X, Y, d)


def plx_spmm_static(ctx: plx_ctx, csr: plx_csr, transposed: bool, X: torch.Tensor, Y: torch.Tensor,
                    d: Optional[int] = None) -> torch.Tensor:
    """plx_spmm / plx_spmm_t through the library's fixed partial-sum buffer: the call allocates nothing."""
    xp, ldx = _mat(X)
    yp, ldy = _mat(Y)
    if d is None:
        d = X.shape[1]
    rows, cols = csr.shape(transposed)
    _check(ctx, "X", X, cols, d); _check(ctx, "Y", Y, rows, d, X.dtype)
    ctx.check(_lib.plx_spmm_static(ctx.handle, csr.handle, int(transposed), xp, ldx, yp, ldy, d, _dtype_code(X)))
    return Y


def plx_gemm_nn(ctx: plx_ctx, A: torch.Tensor, B: torch.Tensor, C: torch.Tensor) -> torch.Tensor:
    """C[M x N] = A[M x K] B[K x N]; B fp32."""
    (ap, lda), (bp, ldb), (cp, ldc) = _mat(A), _mat(B), _mat(C)
    _check(ctx, "B", B, A.shape[1], B.shape[1], torch.float32); _check(ctx, "A", A, A.shape[0], A.shape[1])
    _check(ctx, "C", C, A.shape[0], B.shape[1], A.dtype)
    ctx.check(_lib.plx_gemm_nn(ctx.handle, A.shape[0], B.shape[1], A.shape[1], ap, lda, bp, ldb, cp, ldc, _dtype_code(A)))
    return C


def plx_gemm_nt(ctx: plx_ctx, A: torch.Tensor, B: torch.Tensor, C: torch.Tensor) -> torch.Tensor:
    """C[M x N] = A[M x K] B[N x K]^T; B fp32."""
    (ap, lda), (bp, ldb), (cp, ldc) = _mat(A), _mat(B), _mat(C)
    _check(ctx, "B", B, B.shape[0], A.shape[1], torch.float32); _check(ctx, "A", A, A.shape[0], A.shape[1])
    _check(ctx, "C", C, A.shape[0], B.shape[0], A.dtype)
    ctx.check(_lib.plx_gemm_nt(ctx.handle, A.shape[0], B.shape[0], A.shape[1], ap, lda, bp, ldb, cp, ldc, _dtype_code(A)))
    return C


def plx_gemm_tn_workspace(R: int, M: int, N: int) -> int:
    return int(_lib.plx_gemm_tn_workspace(R, M, N))


def plx_gemm_tn(ctx: plx_ctx, A: torch.Tensor, B: torch.Tensor, C: torch.Tensor, ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """C[M x N] (fp32) = A[R x M]^T B[R x N]."""
    (ap, lda), (bp, ldb), (cp, ldc) = _mat(A), _mat(B), _mat(C)
    R, M, N = A.shape[0], A.shape[1], B.shape[1]
    _check(ctx, "A", A, R, M); _check(ctx, "B", B, R, N, A.dtype); _check(ctx, "C", C, M, N, torch.float32); _check_ws(ctx, ws)
    if ws is None:
        ws = torch.empty(max(1, plx_gemm_tn_workspace(R, M, N)), dtype=torch.uint8, device=A.device)
    ctx.check(_lib.plx_gemm_tn(ctx.handle, R, M, N, ap, lda, bp, ldb, cp, ldc, _dtype_code(A), ws.data_ptr(), ws.numel()))
    return C


def plx_relu(ctx: plx_ctx, Z: torch.Tensor, F: torch.Tensor) -> torch.Tensor:
    (zp, ldz), (fp, ldf) = _mat(Z), _mat(F)
    _check(ctx, "Z", Z, Z.shape[0], Z.shape[1]); _check(ctx, "F", F, Z.shape[0], Z.shape[1], Z.dtype)
    ctx.check(_lib.plx_relu(ctx.handle, Z.shape[0], Z.shape[1], zp, ldz, fp, ldf, _dtype_code(Z)))
    return F


def plx_relu_bwd(ctx: plx_ctx, Z: torch.Tensor, dF: torch.Tensor, dZ: torch.Tensor) -> torch.Tensor:
    (zp, ldz), (gp, ldg), (op, ldo) = _mat(Z), _mat(dF), _mat(dZ)
    _check(ctx, "Z", Z, Z.shape[0], Z.shape[1]); _check(ctx, "dF", dF, Z.shape[0], Z.shape[1], Z.dtype)
    _check(ctx, "dZ", dZ, Z.shape[0], Z.shape[1], Z.dtype)
    ctx.check(_lib.plx_relu_bwd(ctx.handle, Z.shape[0], Z.shape[1], zp, ldz, gp, ldg, op, ldo, _dtype_code(Z)))
    return dZ


def plx_softmax_ce(ctx: plx_ctx, Z: torch.Tensor, y: torch.Tensor, dZ: torch.Tensor,
                   row_loss: Optional[torch.Tensor] = None, loss: Optional[torch.Tensor] = None) -> torch.Tensor:
    (zp, ldz), (gp, ldg) = _mat(Z), _mat(dZ)
    if row_loss is None:
        row_loss = torch.empty(max(1, Z.shape[0]), dtype=torch.float32, device=Z.device)
    _check(ctx, "Z", Z, Z.shape[0], Z.shape[1]); _check(ctx, "dZ", dZ, Z.shape[0], Z.shape[1], Z.dtype)
    for name, t, count in (("y", y, Z.shape[0]), ("row_loss", row_loss, Z.shape[0]), ("loss", loss, 1)):
        if t is not None and (t.numel() < count or (ctx.device >= 0 and (not t.is_cuda or t.device.index != ctx.device))):
            raise ValueError(f"{name}: {t.numel()} elements on {t.device}, the call needs {count} on the context's GPU")
    ctx.check(_lib.plx_softmax_ce(ctx.handle, Z.shape[0], Z.shape[1], zp, ldz, _ptr(y, torch.int64), gp, ldg,
                                  _ptr(row_loss, torch.float32), _ptr(loss, torch.float32), _dtype_code(Z)))
    return dZ


def plx_gcn_layer_plan(ctx: plx_ctx, din: int, dout: int, dn: int = 0, dtype: int = PLX_F32, order: int = PLX_ORDER_AUTO,
                       next_order: int = PLX_ORDER_AUTO, keep_values: bool = False):
    """(agg_first, sign_bits, chain_fwd, chain_bwd) for a layer din -> dout followed (dn > 0) by a layer dout -> dn."""
    out = [_int() for _ in range(4)]
    ctx.check(_lib.plx_gcn_layer_plan(ctx.handle, din, dout, dn, dtype, order, next_order, int(keep_values),
                                      *[ctypes.byref(o) for o in out]))
    return tuple(bool(o.value) for o in out)


def _check_layer(ctx: plx_ctx, csr: plx_csr, transposed_A: bool, din: int, dout: int, tdt, act: int, order: int, dn: int = 0,
                 **ops) -> None:
    """Every tensor of a layer call against the shapes the handle and the widths imply (see _check)."""
    ma, ka = csr.shape(transposed_A)
    agg = plx_gcn_layer_plan(ctx, din, dout, 0, PLX_F32 if tdt == torch.float32 else PLX_BF16, order)[0] if din > 0 and dout > 0 else True
    spec = {"H": (ka, din, tdt), "W": (din, dout, torch.float32), "F": (ma, dout, tdt), "dF": (ma, dout, tdt),
            "saved": (ma if agg else 0, din if agg else 0, tdt), "dH": (ka, din, tdt), "dW": (din, dout, torch.float32),
            "dT": (ka, dout, tdt), "T": (ka, dout, tdt), "Wn": (dout, dn, torch.float32), "Tn": (ma, dn, tdt), "dTn": (ma, dn, tdt),
            "Z": (ma, (dout + 31) // 32, torch.int32) if act == PLX_ACT_RELU_BITS else (ma, dout, tdt)}
    if act not in (PLX_ACT_NONE, PLX_ACT_RELU, PLX_ACT_RELU_BITS):
        ops.pop("Z", None)                                                 # an unknown code is the library's to reject
    for name, t in ops.items():
        if name == "ws":
            _check_ws(ctx, t)
        elif name == "Z" and act == PLX_ACT_RELU and t is not None:       # only the sign is read: any matrix of the layer's type
            _check(ctx, name, t, ma, dout, tdt)
        else:
            _check(ctx, name, t, *spec[name])


def plx_gcn_layer_workspace(csr: plx_csr, transposed_A: bool, din: int, dout: int, dtype: int = PLX_F32,
                            act: int = PLX_ACT_RELU, order: int = PLX_ORDER_AUTO) -> int:
    return int(_lib.plx_gcn_layer_workspace(csr.handle, int(transposed_A), din, dout, dtype, act, order))


def plx_gcn_layer_fwd(ctx: plx_ctx, csr: plx_csr, transposed_A: bool, H: torch.Tensor, W: torch.Tensor,
                      Z: torch.Tensor, F: Optional[torch.Tensor], saved: Optional[torch.Tensor], ws: Optional[torch.Tensor],
                      act: int = PLX_ACT_RELU, order: int = PLX_ORDER_AUTO) -> None:
    (hp, ldh), (wp, ldw), (zp, ldz), (fp, ldf), (sp, lds) = _mat(H), _mat(W), _mat(Z), _mat(F), _mat(saved)
    din, dout = W.shape
    _check_layer(ctx, csr, transposed_A, din, dout, H.dtype, act, order, H=H, W=W, Z=Z, F=F, saved=saved, ws=ws)
    ctx.check(_lib.plx_gcn_layer_fwd(ctx.handle, csr.handle, int(transposed_A), hp, ldh, wp, ldw, din, dout,
                                     _dtype_code(H), act, order, zp, ldz, fp, ldf, sp, lds,
                                     None if ws is None else ws.data_ptr(), 0 if ws is None else ws.numel()))


def plx_gcn_layer_bwd(ctx: plx_ctx, csr: plx_csr, transposed_A: bool, H: Optional[torch.Tensor], W: torch.Tensor,
                      Z: Optional[torch.Tensor], dF: torch.Tensor, saved: Optional[torch.Tensor],
                      dH: Optional[torch.Tensor], dW: torch.Tensor, ws: torch.Tensor,
                      act: int = PLX_ACT_RELU, order: int = PLX_ORDER_AUTO) -> None:
    (hp, ldh), (wp, ldw), (zp, ldz), (gp, ldg), (sp, lds) = _mat(H), _mat(W), _mat(Z), _mat(dF), _mat(saved)
    (dhp, lddh), (dwp, lddw) = _mat(dH), _mat(dW)
    din, dout = W.shape
    _check_layer(ctx, csr, transposed_A, din, dout, dF.dtype, act, order, H=H, W=W, Z=Z, dF=dF, saved=saved, dH=dH, dW=dW, ws=ws)
    ctx.check(_lib.plx_gcn_layer_bwd(ctx.handle, csr.handle, int(transposed_A), hp, ldh, wp, ldw, zp, ldz, gp, ldg,
                                     sp, lds, din, dout, _dtype_code(dF), act, order, dhp, lddh, dwp, lddw,
                                     ws.data_ptr(), ws.numel()))


def plx_gcn_layer_bwd_dt(ctx: plx_ctx, csr: plx_csr, transposed_A: bool, H: torch.Tensor, Z: Optional[torch.Tensor],
                         dF: torch.Tensor, dT: torch.Tensor, dW: torch.Tensor, ws: torch.Tensor,
                         act: int = PLX_ACT_RELU) -> None:
    """Combine-first backward up to dT = A^T (dF * [Z > 0]) and dW = H^T dT; dH = dT W^T is left to the consumer."""
    (hp, ldh), (zp, ldz), (gp, ldg), (tp, ldt), (dwp, lddw) = _mat(H), _mat(Z), _mat(dF), _mat(dT), _mat(dW)
    din, dout = dW.shape
    _check_layer(ctx, csr, transposed_A, din, dout, dF.dtype, act, PLX_ORDER_COMBINE_FIRST, H=H, Z=Z, dF=dF, dT=dT, dW=dW, ws=ws)
    ctx.check(_lib.plx_gcn_layer_bwd_dt(ctx.handle, csr.handle, int(transposed_A), hp, ldh, zp, ldz, gp, ldg, din, dout,
                                        _dtype_code(dF), act, tp, ldt, dwp, lddw, ws.data_ptr(), ws.numel()))


def plx_gcn_layer_bwd_chained_workspace(ctx: plx_ctx, csr: plx_csr, transposed_A: bool, din: int, dout: int, dn: int,
                                        dtype: int = PLX_F32, act: int = PLX_ACT_RELU, order: int = PLX_ORDER_AUTO) -> int:
    return int(_lib.plx_gcn_layer_bwd_chained_workspace(ctx.handle, csr.handle, int(transposed_A), din, dout, dn, dtype, act, order))


def plx_gcn_layer_bwd_chained(ctx: plx_ctx, csr: plx_csr, transposed_A: bool, H: Optional[torch.Tensor], W: torch.Tensor,
                              Z: Optional[torch.Tensor], dTn: torch.Tensor, Wn: torch.Tensor, saved: Optional[torch.Tensor],
                              dH: Optional[torch.Tensor], dW: torch.Tensor, ws: torch.Tensor,
                              act: int = PLX_ACT_RELU, order: int = PLX_ORDER_AUTO) -> None:
    """plx_gcn_layer_bwd with the upstream gradient given as the following layer's (dT, W): dF = dTn Wn^T."""
    (hp, ldh), (wp, ldw), (zp, ldz), (gp, ldg), (wnp, ldwn), (sp, lds) = _mat(H), _mat(W), _mat(Z), _mat(dTn), _mat(Wn), _mat(saved)
    (dhp, lddh), (dwp, lddw) = _mat(dH), _mat(dW)
    din, dout = W.shape
    _check_layer(ctx, csr, transposed_A, din, dout, dTn.dtype, act, order, Wn.shape[1], H=H, W=W, Z=Z, dTn=dTn, Wn=Wn, saved=saved,
                 dH=dH, dW=dW, ws=ws)
    ctx.check(_lib.plx_gcn_layer_bwd_chained(ctx.handle, csr.handle, int(transposed_A), hp, ldh, wp, ldw, zp, ldz, gp, ldg,
                                             wnp, ldwn, Wn.shape[1], sp, lds, din, dout, _dtype_code(dTn), act, order,
                                             dhp, lddh, dwp, lddw, ws.data_ptr(), ws.numel()))


def plx_gcn_layer_fwd_chained(ctx: plx_ctx, csr: plx_csr, transposed_A: bool, H: torch.Tensor, W: torch.Tensor,
                              Z: Optional[torch.Tensor], F: Optional[torch.Tensor], saved: Optional[torch.Tensor],
                              Wn: torch.Tensor, Tn: torch.Tensor, ws: Optional[torch.Tensor],
                              act: int = PLX_ACT_RELU, order: int = PLX_ORDER_AUTO) -> None:
    """plx_gcn_layer_fwd that also writes Tn = (this layer's output) Wn, the first product of a following combine-first layer."""
    (hp, ldh), (wp, ldw), (zp, ldz), (fp, ldf), (sp, lds) = _mat(H), _mat(W), _mat(Z), _mat(F), _mat(saved)
    (wnp, ldwn), (tp, ldt) = _mat(Wn), _mat(Tn)
    din, dout = W.shape
    _check_layer(ctx, csr, transposed_A, din, dout, H.dtype, act, order, Wn.shape[1], H=H, W=W, Z=Z, F=F, saved=saved, Wn=Wn, Tn=Tn,
                 ws=ws)
    ctx.check(_lib.plx_gcn_layer_fwd_chained(ctx.handle, csr.handle, int(transposed_A), hp, ldh, wp, ldw, din, dout,
                                             _dtype_code(H), act, order, zp, ldz, fp, ldf, sp, lds, wnp, ldwn, Wn.shape[1], tp, ldt,
                                             None if ws is None else ws.data_ptr(), 0 if ws is None else ws.numel()))


def plx_gcn_layer_fwd_from_t(ctx: plx_ctx, csr: plx_csr, transposed_A: bool, T: torch.Tensor, Z: Optional[torch.Tensor],
                             F: Optional[torch.Tensor], act: int = PLX_ACT_RELU) -> None:
    """Z = A T, F = act(Z): a combine-first layer whose T = H W already exists."""
    (tp, ldt), (zp, ldz), (fp, ldf) = _mat(T), _mat(Z), _mat(F)
    _check_layer(ctx, csr, transposed_A, T.shape[1], T.shape[1], T.dtype, act, PLX_ORDER_COMBINE_FIRST, T=T, Z=Z, F=F)
    ctx.check(_lib.plx_gcn_layer_fwd_from_t(ctx.handle, csr.handle, int(transposed_A), tp, ldt, T.shape[1], _dtype_code(T), act,
                                            zp, ldz, fp, ldf))
