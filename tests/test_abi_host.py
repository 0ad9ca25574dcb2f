"""Host-side checks that need no GPU: the shared library loads, exports every symbol the
header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest
import torch

import paper_2505_04083_amd as plx

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "plx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"PLX_API[^;(]*?\b(plx_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 20
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2505_04083_amd", "libplx.so"))
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(plx.EXPORTED) == names


@pytest.fixture(scope="module")
def dry():
    ctx = plx.plx_ctx(device=-1)
    yield ctx
    ctx.close()


def expect(status, fn, *a, **k):
    with pytest.raises(plx.PlxError) as e:
        fn(*a, **k)
    assert e.value.status == status, str(e.value)


def test_context_errors():
    out = ctypes.c_void_p()
    assert plx._lib.plx_ctx_create(-2, None, plx._ALLOC_FN(0), plx._FREE_FN(0), None, ctypes.byref(out)) == plx.PLX_ERR_INVALID
    assert plx._lib.plx_ctx_create(0, None, plx._ALLOC_FN(0), plx._FREE_FN(0), None, None) == plx.PLX_ERR_INVALID
    if not torch.cuda.is_available():
        # no GPU here: a clean status, not an abort
        assert plx._lib.plx_ctx_create(0, None, plx._ALLOC_FN(0), plx._FREE_FN(0), None, ctypes.byref(out)) == plx.PLX_ERR_DEVICE
    assert plx._lib.plx_status_string(plx.PLX_ERR_SHAPE) == b"shape mismatch"
    assert plx._lib.plx_sync(None) == plx.PLX_ERR_INVALID


def test_build_csr_argument_checks(dry):
    e = torch.zeros(4, dtype=torch.int64)
    expect(plx.PLX_ERR_INVALID, plx.plx_build_csr, dry, -1, e, e)
    out = ctypes.c_void_p()
    L = plx._lib
    assert L.plx_build_csr(dry.handle, 10, 4, None, e.data_ptr(), None, None, ctypes.byref(out)) == plx.PLX_ERR_INVALID
    assert L.plx_build_csr(dry.handle, 10, 4, e.data_ptr(), e.data_ptr(), None, None, None) == plx.PLX_ERR_INVALID
    assert L.plx_build_csr(dry.handle, 1 << 31, 0, None, None, None, None, ctypes.byref(out)) == plx.PLX_ERR_UNSUPPORTED
    assert L.plx_build_csr(None, 10, 0, None, None, None, None, ctypes.byref(out)) == plx.PLX_ERR_INVALID
    # valid arguments on a validate-only context: refused with the device status, nothing ran
    expect(plx.PLX_ERR_DEVICE, plx.plx_build_csr, dry, 10, e, e)
    assert b"validate-only" in L.plx_last_error(dry.handle)
    rp = torch.zeros(3, dtype=torch.int64); c = torch.zeros(1, dtype=torch.int32); v = torch.zeros(1)
    assert L.plx_csr_import(dry.handle, 2, 2, 1, None, c.data_ptr(), v.data_ptr(), ctypes.byref(out)) == plx.PLX_ERR_INVALID
    assert L.plx_csr_import(dry.handle, -2, 2, 1, rp.data_ptr(), c.data_ptr(), v.data_ptr(), ctypes.byref(out)) == plx.PLX_ERR_INVALID
    expect(plx.PLX_ERR_DEVICE, plx.plx_csr_import, dry, 2, 2, rp, c, v)


def test_dense_and_elementwise_argument_checks(dry):
    L = plx._lib
    A = torch.zeros(8, 4); B = torch.zeros(4, 6); C = torch.zeros(8, 6)
    expect(plx.PLX_ERR_DEVICE, plx.plx_gemm_nn, dry, A, B, C)
    h = dry.handle
    p = A.data_ptr()
    assert L.plx_gemm_nn(h, 8, 6, 4, p, 3, B.data_ptr(), 6, C.data_ptr(), 6, 0) == plx.PLX_ERR_SHAPE     # lda < K
    assert L.plx_gemm_nn(h, 8, 6, 4, p, 4, B.data_ptr(), 5, C.data_ptr(), 6, 0) == plx.PLX_ERR_SHAPE     # ldb < N
    assert L.plx_gemm_nt(h, 8, 6, 4, p, 4, B.data_ptr(), 3, C.data_ptr(), 6, 0) == plx.PLX_ERR_SHAPE     # ldb < K
    assert L.plx_gemm_nn(h, 8, 6, 4, None, 4, B.data_ptr(), 6, C.data_ptr(), 6, 0) == plx.PLX_ERR_INVALID
    assert L.plx_gemm_nn(h, -1, 6, 4, p, 4, B.data_ptr(), 6, C.data_ptr(), 6, 0) == plx.PLX_ERR_INVALID
    assert L.plx_gemm_nn(h, 8, 6, 4, p, 4, B.data_ptr(), 6, C.data_ptr(), 6, 7) == plx.PLX_ERR_INVALID   # dtype
    need = L.plx_gemm_tn_workspace(8, 4, 6)
    assert need >= 4 * 6 * 4
    assert L.plx_gemm_tn(h, 8, 4, 6, p, 4, C.data_ptr(), 6, B.data_ptr(), 6, 0, p, need - 1) == plx.PLX_ERR_SHAPE
    assert L.plx_relu(h, 8, 4, p, 3, p, 4, 0) == plx.PLX_ERR_SHAPE
    assert L.plx_relu_bwd(h, 8, 4, p, 4, None, 4, p, 4, 0) == plx.PLX_ERR_INVALID
    y = torch.zeros(8, dtype=torch.int64)
    assert L.plx_softmax_ce(h, 8, 0, p, 4, y.data_ptr(), p, 4, p, None, 0) == plx.PLX_ERR_INVALID
    assert L.plx_softmax_ce(h, 8, 4, p, 4, y.data_ptr(), p, 4, p, None, 0) == plx.PLX_ERR_DEVICE
    assert L.plx_spmm(h, None, p, 4, p, 4, 4, 0) == plx.PLX_ERR_INVALID                                  # no handle
    assert L.plx_gcn_layer_fwd(h, None, 0, p, 4, p, 4, 4, 4, 0, 1, 0, p, 4, None, 0, None, 0, None, 0) == plx.PLX_ERR_INVALID
    assert L.plx_gcn_layer_workspace(None, 0, 4, 4, 0, 1, 0) == 0
    # the layer-pair calls: no handle, no context, missing outputs
    assert L.plx_gcn_layer_fwd_chained(h, None, 0, p, 4, p, 4, 4, 4, 0, 1, 0, p, 4, p, 4, p, 4, p, 4, 4, p, 4, None, 0) == plx.PLX_ERR_INVALID
    assert L.plx_gcn_layer_fwd_chained(h, None, 0, p, 4, p, 4, 4, 4, 0, 1, 0, p, 4, p, 4, p, 4, p, 4, 4, None, 4, None, 0) == plx.PLX_ERR_INVALID
    assert b"Tn is NULL" in L.plx_last_error(h)
    assert L.plx_gcn_layer_fwd_from_t(h, None, 0, p, 4, 4, 0, 1, p, 4, None, 0) == plx.PLX_ERR_INVALID
    assert L.plx_gcn_layer_fwd_from_t(h, None, 0, None, 4, 4, 0, 1, p, 4, None, 0) == plx.PLX_ERR_INVALID
    assert b"T is NULL" in L.plx_last_error(h)
    assert L.plx_gcn_layer_bwd_dt(h, None, 0, p, 4, None, 0, p, 4, 4, 4, 0, 0, p, 4, p, 4, p, 64) == plx.PLX_ERR_INVALID
    assert L.plx_gcn_layer_bwd_dt(h, None, 0, p, 4, None, 0, p, 4, 4, 4, 0, 0, None, 4, p, 4, p, 64) == plx.PLX_ERR_INVALID
    assert b"dT is NULL" in L.plx_last_error(h)
    assert L.plx_gcn_layer_bwd_chained(h, None, 0, p, 4, p, 4, None, 0, p, 4, p, 4, 4, p, 4, 4, 4, 0, 0, 0, p, 4, p, 4, p, 64) == plx.PLX_ERR_INVALID
    assert L.plx_gcn_layer_bwd_chained(None, None, 0, p, 4, p, 4, None, 0, p, 4, p, 4, 4, p, 4, 4, 4, 0, 0, 0, p, 4, p, 4, p, 64) == plx.PLX_ERR_INVALID
    assert L.plx_gcn_layer_bwd_chained_workspace(h, None, 0, 4, 4, 4, 0, 1, 0) == 0
    assert L.plx_csr_dims(None, None, None, None) == plx.PLX_ERR_INVALID
    # tuning knob and blocked aggregation: argument rules hold without a device
    assert L.plx_ctx_set_column_windows(h, 0) == plx.PLX_ERR_INVALID
    assert L.plx_ctx_set_column_windows(h, 65) == plx.PLX_ERR_INVALID
    assert L.plx_ctx_set_column_windows(h, 8) == plx.PLX_OK
    assert L.plx_ctx_set_column_windows(None, 8) == plx.PLX_ERR_INVALID
    assert L.plx_ctx_set_split_products(h, 0) == plx.PLX_OK and L.plx_ctx_set_split_products(h, 1) == plx.PLX_OK
    assert L.plx_ctx_set_split_products(None, 1) == plx.PLX_ERR_INVALID
    assert L.plx_csr_set_row_blocks(h, None, 4) == plx.PLX_ERR_INVALID
    assert L.plx_spmm_block(h, None, 0, 0, p, 4, p, 4, 4, 0) == plx.PLX_ERR_INVALID
