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


# ---- the binding's own checks: what the C side cannot see (device, element type, extent of a tensor) ------------

class FakeHandle:
    """Stands in for an adjacency handle: the binding reads only its shape before it validates the tensors."""
    handle = None

    def __init__(self, m, k):
        self.m, self.k = m, k

    def shape(self, transposed=False):
        return (self.k, self.m) if transposed else (self.m, self.k)


class OnGpu0:
    """A context that claims GPU 0 (no call reaches the library with it)."""
    device = 0
    handle = None


def test_binding_rejects_wrong_shaped_or_typed_tensors(dry):
    csr = FakeHandle(10, 20)
    X = torch.zeros(20, 8); Y = torch.zeros(10, 8)
    with pytest.raises(ValueError, match="X: shape"):
        plx.plx_spmm(dry, csr, torch.zeros(19, 8), Y)                    # X shorter than the handle's column count
    with pytest.raises(ValueError, match="Y: shape"):
        plx.plx_spmm(dry, csr, X, torch.zeros(9, 8))
    with pytest.raises(ValueError, match="Y: shape"):
        plx.plx_spmm_t(dry, csr, torch.zeros(10, 8), torch.zeros(10, 8))  # transposed: Y has the handle's 20 columns as rows
    with pytest.raises(TypeError, match="Y: expected"):
        plx.plx_spmm(dry, csr, X.bfloat16(), Y)                           # one element type per call
    with pytest.raises(ValueError, match="Y: shape"):
        plx.plx_spmm_static(dry, csr, False, X, torch.zeros(10, 4))
    with pytest.raises(ValueError, match="C: shape"):
        plx.plx_gemm_nn(dry, torch.zeros(8, 4), torch.zeros(4, 6), torch.zeros(8, 5))
    with pytest.raises(TypeError, match="B: expected"):
        plx.plx_gemm_nn(dry, torch.zeros(8, 4), torch.zeros(4, 6).bfloat16(), torch.zeros(8, 6))
    with pytest.raises(ValueError, match="y:"):
        plx.plx_softmax_ce(dry, torch.zeros(8, 4), torch.zeros(7, dtype=torch.int64), torch.zeros(8, 4))
    # a layer: every operand against the handle and the widths
    W = torch.zeros(8, 16); H = torch.zeros(20, 8); F = torch.zeros(10, 16); saved = torch.zeros(10, 8)
    ws = torch.zeros(64, dtype=torch.uint8)
    with pytest.raises(ValueError, match="H: shape"):
        plx.plx_gcn_layer_fwd(dry, csr, False, torch.zeros(10, 8), W, None, F, saved, ws)
    with pytest.raises(ValueError, match="saved: shape"):
        plx.plx_gcn_layer_fwd(dry, csr, False, H, W, None, F, torch.zeros(1, 8), ws, order=plx.PLX_ORDER_AGG_FIRST)
    with pytest.raises(TypeError, match="Z: expected torch.int32"):
        plx.plx_gcn_layer_fwd(dry, csr, False, H, W, torch.zeros(10, 1), F, saved, ws, act=plx.PLX_ACT_RELU_BITS)
    with pytest.raises(TypeError, match="F: expected"):
        plx.plx_gcn_layer_fwd(dry, csr, False, H, W, None, F.bfloat16(), saved, ws)
    with pytest.raises(ValueError, match="dH: shape"):
        plx.plx_gcn_layer_bwd(dry, csr, False, H, W, F, torch.zeros(10, 16), saved, torch.zeros(10, 8), torch.zeros(8, 16), ws)
    with pytest.raises(TypeError, match="workspace"):
        plx.plx_gcn_layer_bwd(dry, csr, False, H, W, F, torch.zeros(10, 16), saved, torch.zeros(20, 8), torch.zeros(8, 16),
                              torch.zeros(64))
    with pytest.raises(ValueError, match="dTn: shape"):
        plx.plx_gcn_layer_bwd_chained(dry, csr, False, H, W, None, torch.zeros(9, 4), torch.zeros(16, 4), saved, torch.zeros(20, 8),
                                      torch.zeros(8, 16), ws, act=plx.PLX_ACT_NONE)
    with pytest.raises(ValueError, match="T: shape"):
        plx.plx_gcn_layer_fwd_from_t(dry, csr, False, torch.zeros(19, 16), None, F, act=plx.PLX_ACT_NONE)
    # a combine-first layer never reads `saved`: a placeholder of any size passes the binding (and reaches the C checks)
    expect(plx.PLX_ERR_DEVICE, plx.plx_gemm_nn, dry, torch.zeros(8, 4), torch.zeros(4, 6), torch.zeros(8, 6))


def test_binding_rejects_tensors_on_another_device():
    with pytest.raises(ValueError, match="the context runs on cuda:0"):
        plx._check(OnGpu0(), "X", torch.zeros(4, 4), 4, 4)
    with pytest.raises(ValueError, match="workspace on cpu"):
        plx._check_ws(OnGpu0(), torch.zeros(4, dtype=torch.uint8))


def test_layer_plan_without_a_device(dry):
    """The sequencer's questions are answered on the host: no device needed, one place for the kernels' shape limits."""
    assert plx.plx_gcn_layer_plan(dry, 64, 128, 16) == (True, True, True, True)           # the road network's pair
    assert plx.plx_gcn_layer_plan(dry, 64, 128, 16, keep_values=True) == (True, False, True, False)
    assert plx.plx_gcn_layer_plan(dry, 128, 128, 47) == (True, True, False, False)         # wide factor: not worth forming in the kernel
    assert plx.plx_gcn_layer_plan(dry, 602, 128, 16) == (False, False, False, False)       # combine-first layer
    assert plx.plx_gcn_layer_plan(dry, 32, 128, 16) == (True, True, False, False)          # narrow input: fp32 instructions, no pairing
    assert plx.plx_gcn_layer_plan(dry, 64, 128, 16, dtype=plx.PLX_BF16) == (True, True, False, False)
    assert plx.plx_gcn_layer_plan(dry, 64, 128, 16, next_order=plx.PLX_ORDER_AGG_FIRST)[2:] == (False, False)
    plx.plx_ctx_set_split_products(dry, False)
    assert plx.plx_gcn_layer_plan(dry, 64, 128, 16) == (True, True, False, False)          # the pairing lives in the split kernels
    plx.plx_ctx_set_split_products(dry, True)
    assert plx._lib.plx_gcn_layer_plan(dry.handle, 0, 128, 16, 0, 2, 2, 0, None, None, None, None) == plx.PLX_ERR_INVALID
    assert plx._lib.plx_gcn_layer_plan(None, 64, 128, 16, 0, 2, 2, 0, None, None, None, None) == plx.PLX_ERR_INVALID
