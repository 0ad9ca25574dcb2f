// C-ABI entry points: argument validation, context, handle bookkeeping and the composition
// of one GCN layer (paper Sec. 2.1, Eq. 2.1-2.7) out of the kernels in the other files.
#include "plx_internal.h"

#include <algorithm>
#include <cstring>

namespace plx {

plx_status fail(plx_ctx* ctx, plx_status s, const char* fmt, ...) {
    if (ctx) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        ctx->err = buf;
    }
    return s;
}

void* dev_alloc(plx_ctx* ctx, size_t bytes) {
    if (bytes == 0) bytes = 256;
    void* p = nullptr;
    if (ctx->alloc) {
        p = ctx->alloc(bytes, ctx->user);
    } else if (hipMalloc(&p, bytes) != hipSuccess) {
        (void)hipGetLastError();
        p = nullptr;
    }
    if (!p) fail(ctx, PLX_ERR_OOM, "device allocation of %zu bytes failed", bytes);
    return p;
}

void dev_free(plx_ctx* ctx, void* p) {
    if (!p) return;
    if (ctx->release) ctx->release(p, ctx->user);
    else (void)hipFree(p);
}

void free_orient(plx_ctx* ctx, Orient& o) {
    dev_free(ctx, o.rowptr); dev_free(ctx, o.col); dev_free(ctx, o.val); dev_free(ctx, o.row_order);
    dev_free(ctx, o.bptr);
    dev_free(ctx, o.long_row); dev_free(ctx, o.long_seg0); dev_free(ctx, o.seg_lo); dev_free(ctx, o.seg_len);
    dev_free(ctx, o.seg_launch); dev_free(ctx, o.part); dev_free(ctx, o.seg_desc);
    o = Orient();
}

static bool dtype_ok(plx_dtype t) { return t == PLX_F32 || t == PLX_BF16; }

}  // namespace plx

using namespace plx;

extern "C" {

const char* plx_status_string(plx_status s) {
    switch (s) {
        case PLX_OK: return "ok";
        case PLX_ERR_INVALID: return "invalid argument";
        case PLX_ERR_SHAPE: return "shape mismatch";
        case PLX_ERR_UNSUPPORTED: return "unsupported";
        case PLX_ERR_OOM: return "out of device memory";
        case PLX_ERR_DEVICE: return "device error";
        case PLX_ERR_INTERNAL: return "internal error";
    }
    return "unknown status";
}

plx_status plx_ctx_create(int device, void* hip_stream, plx_alloc_fn alloc, plx_free_fn release, void* user,
                          plx_ctx** out) {
    if (!out) return PLX_ERR_INVALID;
    *out = nullptr;
    if (device < -1) return PLX_ERR_INVALID;
    if ((alloc == nullptr) != (release == nullptr)) return PLX_ERR_INVALID;
    plx_ctx* c = new (std::nothrow) plx_ctx();
    if (!c) return PLX_ERR_OOM;
    c->device = device;
    c->dry = device == -1;
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->alloc = alloc; c->release = release; c->user = user;
    if (!c->dry) {
        int count = 0;
        if (hipGetDeviceCount(&count) != hipSuccess || device >= count) {
            (void)hipGetLastError();
            delete c;
            return PLX_ERR_DEVICE;
        }
        if (hipSetDevice(device) != hipSuccess) {
            (void)hipGetLastError();
            delete c;
            return PLX_ERR_DEVICE;
        }
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && cus > 0) c->n_cu = cus;
        // the fixed buffer of plx_spmm_static: its address on this GPU is looked up here, once, so that the call
        // itself does no set-up work; a failure is reported by that call, not by this one
        (void)static_partials(c, nullptr);
    }

    *out = c;
    return PLX_OK;
}

void plx_ctx_destroy(plx_ctx* ctx) {
    if (!ctx) return;
    if (!ctx->dry) (void)hipStreamSynchronize(ctx->stream);
    for (auto& t : ctx->timed) { (void)hipEventDestroy(t.start); (void)hipEventDestroy(t.stop); }
    delete ctx;
}

plx_status plx_ctx_set_split_products(plx_ctx* ctx, int on) {
    if (!ctx) return PLX_ERR_INVALID;
    ctx->split_products = on != 0;
    return PLX_OK;
}

plx_status plx_ctx_set_fused_aggregation(plx_ctx* ctx, int on) {
    if (!ctx) return PLX_ERR_INVALID;
    ctx->fused_aggregation = on != 0;
    return PLX_OK;
}

plx_status plx_ctx_set_column_windows(plx_ctx* ctx, int n_windows) {
    if (!ctx) return PLX_ERR_INVALID;
    if (n_windows < 1 || n_windows > 64) return fail(ctx, PLX_ERR_INVALID, "n_windows must be between 1 and 64");
    ctx->n_windows = n_windows;
    return PLX_OK;
}

const char* plx_last_error(const plx_ctx* ctx) { return ctx ? ctx->err.c_str() : "no context"; }

plx_status plx_sync(plx_ctx* ctx) {
    if (!ctx) return PLX_ERR_INVALID;
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");
    PLX_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return PLX_OK;
}

plx_status plx_csr_dims(const plx_csr* csr, int64_t* m, int64_t* k, int64_t* nnz) {
    if (!csr) return PLX_ERR_INVALID;
    if (m) *m = csr->o[0].rows;
    if (k) *k = csr->o[0].cols;
    if (nnz) *nnz = csr->o[0].nnz;
    return PLX_OK;
}

plx_status plx_csr_export(plx_ctx* ctx, const plx_csr* csr, int transposed, int64_t* rowptr, int32_t* col,
                          float* val, int64_t* deg) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!csr) return fail(ctx, PLX_ERR_INVALID, "csr is NULL");
    if (deg && !csr->deg) return fail(ctx, PLX_ERR_INVALID, "this handle holds no degrees (made by plx_csr_import)");
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");
    const Orient& o = csr->o[transposed ? 1 : 0];
    if (rowptr) PLX_HIP(ctx, hipMemcpyAsync(rowptr, o.rowptr, sizeof(int64_t) * (o.rows + 1), hipMemcpyDeviceToDevice, ctx->stream));
    PLX_TRY(export_entries(ctx, o, col, val));
    if (deg && csr->n_deg) PLX_HIP(ctx, hipMemcpyAsync(deg, csr->deg, sizeof(int64_t) * csr->n_deg, hipMemcpyDeviceToDevice, ctx->stream));
    PLX_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return PLX_OK;
}

void plx_csr_destroy(plx_ctx* ctx, plx_csr* csr) {
    if (!ctx || !csr) return;
    if (!ctx->dry) (void)hipStreamSynchronize(ctx->stream);
    free_orient(ctx, csr->o[0]);
    free_orient(ctx, csr->o[1]);
    dev_free(ctx, csr->deg);
    delete csr;
}

plx_status plx_csr_bins(const plx_csr* csr, int transposed, int64_t* rows, int64_t* entries) {
    if (!csr) return PLX_ERR_INVALID;
    const Orient& o = csr->o[transposed ? 1 : 0];
    const int edge[4] = {0, kSubwaveMaxClass + 1, kLongClass, kNumClasses};
    for (int b = 0; b < 3; ++b) {
        int64_t nz = 0, nr = 0;
        for (int blk = 0; blk < o.n_blocks; ++blk) {
            for (int c = edge[b]; c < edge[b + 1]; ++c) nz += o.bnnz[(size_t)blk * kNumClasses + c];
            nr += o.off(blk, edge[b + 1]) - o.off(blk, edge[b]);
        }
        if (rows) rows[b] = nr;
        if (entries) entries[b] = nz;
    }
    return PLX_OK;
}

plx_status plx_timing_enable(plx_ctx* ctx, int on) {
    if (!ctx) return PLX_ERR_INVALID;
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");
    ctx->timing = on != 0;
    return PLX_OK;
}

plx_status plx_timing_report(plx_ctx* ctx, char* buf, size_t buf_bytes) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!buf || buf_bytes == 0) return fail(ctx, PLX_ERR_INVALID, "buf is NULL or empty");
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");
    PLX_HIP(ctx, hipStreamSynchronize(ctx->stream));
    std::vector<std::string> names;
    std::vector<double> total;
    std::vector<long> count;
    for (auto& t : ctx->timed) {
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, t.start, t.stop);
        (void)hipEventDestroy(t.start);
        (void)hipEventDestroy(t.stop);
        size_t i = 0;
        while (i < names.size() && names[i] != t.name) ++i;
        if (i == names.size()) { names.push_back(t.name); total.push_back(0.0); count.push_back(0); }
        total[i] += ms; count[i] += 1;
    }
    ctx->timed.clear();
    std::string out;
    for (size_t i = 0; i < names.size(); ++i) {
        char line[256];
        snprintf(line, sizeof line, "%s %ld %.6f\n", names[i].c_str(), count[i], total[i]);
        out += line;
    }
    size_t n = std::min(out.size(), buf_bytes - 1);
    memcpy(buf, out.data(), n);
    buf[n] = 0;
    return PLX_OK;
}

plx_status plx_timing_trace(plx_ctx* ctx, char* buf, size_t buf_bytes) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!buf || buf_bytes == 0) return fail(ctx, PLX_ERR_INVALID, "buf is NULL or empty");
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");
    PLX_HIP(ctx, hipStreamSynchronize(ctx->stream));
    std::string out;
    for (auto& t : ctx->timed) {
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, t.start, t.stop);
        (void)hipEventDestroy(t.start);
        (void)hipEventDestroy(t.stop);
        char line[256];
        snprintf(line, sizeof line, "%s %.6f\n", t.name.c_str(), ms);
        out += line;
    }
    ctx->timed.clear();
    if (out.size() + 1 > buf_bytes)
        return fail(ctx, PLX_ERR_SHAPE, "the trace takes %zu bytes, the buffer holds %zu (the record was cleared)", out.size() + 1, buf_bytes);
    memcpy(buf, out.data(), out.size());
    buf[out.size()] = 0;
    return PLX_OK;
}

// ---- sparse x dense ---------------------------------------------------------------------------

static plx_status spmm_entry(plx_ctx* ctx, const plx_csr* csr, int t, const void* X, int64_t ldx, void* Y,
                             int64_t ldy, int64_t d, plx_dtype dtype) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!csr) return fail(ctx, PLX_ERR_INVALID, "csr is NULL");
    if (!dtype_ok(dtype)) return fail(ctx, PLX_ERR_INVALID, "unknown dtype %d", (int)dtype);
    if (d < 0) return fail(ctx, PLX_ERR_INVALID, "d = %lld is negative", (long long)d);
    const Orient& o = csr->o[t];
    if (d > 0 && ((o.cols > 0 && !X) || (o.rows > 0 && !Y))) return fail(ctx, PLX_ERR_INVALID, "X or Y is NULL");
    if (ldx < d || ldy < d) return fail(ctx, PLX_ERR_SHAPE, "leading dimension (%lld, %lld) smaller than d = %lld",
                                        (long long)ldx, (long long)ldy, (long long)d);
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");
    if (d == 0 || o.rows == 0) return PLX_OK;
    return launch_spmm(ctx, o, X, ldx, Y, ldy, d, dtype);
}

plx_status plx_csr_row_blocks(const plx_csr* csr, int transposed, int* n_blocks, int64_t* rows_per_block) {
    if (!csr) return PLX_ERR_INVALID;
    const Orient& o = csr->o[transposed ? 1 : 0];
    if (n_blocks) *n_blocks = o.n_blocks;
    if (rows_per_block) *rows_per_block = o.rows_per_block;
    return PLX_OK;
}

plx_status plx_spmm_block(plx_ctx* ctx, const plx_csr* csr, int transposed, int block, const void* X, int64_t ldx,
                          void* Y, int64_t ldy, int64_t d, plx_dtype dtype) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!csr) return fail(ctx, PLX_ERR_INVALID, "csr is NULL");
    const Orient& o = csr->o[transposed ? 1 : 0];
    if (block < 0 || block >= o.n_blocks) return fail(ctx, PLX_ERR_INVALID, "block %d outside [0, %d)", block, o.n_blocks);
    if (!dtype_ok(dtype)) return fail(ctx, PLX_ERR_INVALID, "unknown dtype %d", (int)dtype);
    if (d < 0) return fail(ctx, PLX_ERR_INVALID, "d = %lld is negative", (long long)d);
    if (d > 0 && ((o.cols > 0 && !X) || (o.rows > 0 && !Y))) return fail(ctx, PLX_ERR_INVALID, "X or Y is NULL");
    if (ldx < d || ldy < d) return fail(ctx, PLX_ERR_SHAPE, "leading dimension smaller than d");
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");
    if (d == 0 || o.rows == 0) return PLX_OK;
    return launch_spmm(ctx, o, X, ldx, Y, ldy, d, dtype, nullptr, 0, block);
}

plx_status plx_spmm_static(plx_ctx* ctx, const plx_csr* csr, int transposed, const void* X, int64_t ldx, void* Y,
                           int64_t ldy, int64_t d, plx_dtype dtype) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!csr) return fail(ctx, PLX_ERR_INVALID, "csr is NULL");
    if (!dtype_ok(dtype)) return fail(ctx, PLX_ERR_INVALID, "unknown dtype %d", (int)dtype);
    if (d < 0) return fail(ctx, PLX_ERR_INVALID, "d = %lld is negative", (long long)d);
    const Orient& o = csr->o[transposed ? 1 : 0];
    if (d > 0 && ((o.cols > 0 && !X) || (o.rows > 0 && !Y))) return fail(ctx, PLX_ERR_INVALID, "X or Y is NULL");
    if (ldx < d || ldy < d) return fail(ctx, PLX_ERR_SHAPE, "leading dimension (%lld, %lld) smaller than d = %lld",
                                        (long long)ldx, (long long)ldy, (long long)d);
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");
    if (d == 0 || o.rows == 0) return PLX_OK;
    size_t bytes = 0;
    float* part = static_partials(ctx, &bytes);    // a table look-up after plx_ctx_create
    if (!part) return fail(ctx, PLX_ERR_DEVICE, "the address of the fixed partial-sum buffer could not be obtained on device %d", ctx->device);
    return launch_spmm(ctx, o, X, ldx, Y, ldy, d, dtype, nullptr, 0, -1, part, bytes);
}

plx_status plx_spmm(plx_ctx* ctx, const plx_csr* csr, const void* X, int64_t ldx, void* Y, int64_t ldy, int64_t d,
                    plx_dtype dtype) {
    return spmm_entry(ctx, csr, 0, X, ldx, Y, ldy, d, dtype);
}

plx_status plx_spmm_t(plx_ctx* ctx, const plx_csr* csr, const void* X, int64_t ldx, void* Y, int64_t ldy, int64_t d,
                      plx_dtype dtype) {
    return spmm_entry(ctx, csr, 1, X, ldx, Y, ldy, d, dtype);
}

// ---- dense x dense ----------------------------------------------------------------------------

static plx_status gemm_entry(plx_ctx* ctx, bool bt, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                             const float* B, int64_t ldb, void* C, int64_t ldc, plx_dtype dtype) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!dtype_ok(dtype)) return fail(ctx, PLX_ERR_INVALID, "unknown dtype %d", (int)dtype);
    if (M < 0 || N < 0 || K < 0) return fail(ctx, PLX_ERR_INVALID, "negative dimension");
    if (M > 0 && N > 0 && (!C || (K > 0 && (!A || !B)))) return fail(ctx, PLX_ERR_INVALID, "A, B or C is NULL");
    if (lda < K || ldc < N || ldb < (bt ? K : N)) return fail(ctx, PLX_ERR_SHAPE, "leading dimension too small");
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");
    if (M == 0 || N == 0) return PLX_OK;
    return launch_gemm(ctx, bt, M, N, K, A, lda, B, ldb, C, ldc, dtype);
}

plx_status plx_gemm_nn(plx_ctx* ctx, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const float* B,
                       int64_t ldb, void* C, int64_t ldc, plx_dtype dtype) {
    return gemm_entry(ctx, false, M, N, K, A, lda, B, ldb, C, ldc, dtype);
}

plx_status plx_gemm_nt(plx_ctx* ctx, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const float* B,
                       int64_t ldb, void* C, int64_t ldc, plx_dtype dtype) {
    return gemm_entry(ctx, true, M, N, K, A, lda, B, ldb, C, ldc, dtype);
}

size_t plx_gemm_tn_workspace(int64_t R, int64_t M, int64_t N) {
    if (R < 0 || M <= 0 || N <= 0) return 0;
    return gemm_tn_workspace(R, M, N);
}

plx_status plx_gemm_tn(plx_ctx* ctx, int64_t R, int64_t M, int64_t N, const void* A, int64_t lda, const void* B,
                       int64_t ldb, float* C, int64_t ldc, plx_dtype dtype, void* ws, size_t ws_bytes) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!dtype_ok(dtype)) return fail(ctx, PLX_ERR_INVALID, "unknown dtype %d", (int)dtype);
    if (R < 0 || M < 0 || N < 0) return fail(ctx, PLX_ERR_INVALID, "negative dimension");
    if (M > 0 && N > 0 && (!C || (R > 0 && (!A || !B)))) return fail(ctx, PLX_ERR_INVALID, "A, B or C is NULL");
    if (lda < M || ldb < N || ldc < N) return fail(ctx, PLX_ERR_SHAPE, "leading dimension too small");
    if (M > 0 && N > 0 && (ws_bytes < gemm_tn_workspace(R, M, N) || !ws))
        return fail(ctx, PLX_ERR_SHAPE, "workspace of %zu bytes is smaller than the %zu needed", ws_bytes,
                    gemm_tn_workspace(R, M, N));
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");
    if (M == 0 || N == 0) return PLX_OK;
    return launch_gemm_tn(ctx, R, M, N, A, lda, B, ldb, C, ldc, dtype, ws, ws_bytes);
}

// ---- element-wise ------------------------------------------------------------------------------

plx_status plx_relu(plx_ctx* ctx, int64_t rows, int64_t cols, const void* Z, int64_t ldz, void* F, int64_t ldf,
                    plx_dtype dtype) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!dtype_ok(dtype)) return fail(ctx, PLX_ERR_INVALID, "unknown dtype %d", (int)dtype);
    if (rows < 0 || cols < 0) return fail(ctx, PLX_ERR_INVALID, "negative dimension");
    if (rows > 0 && cols > 0 && (!Z || !F)) return fail(ctx, PLX_ERR_INVALID, "Z or F is NULL");
    if (ldz < cols || ldf < cols) return fail(ctx, PLX_ERR_SHAPE, "leading dimension too small");
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");
    if (rows == 0 || cols == 0) return PLX_OK;
    return launch_relu(ctx, rows, cols, Z, ldz, F, ldf, dtype);
}

plx_status plx_relu_bwd(plx_ctx* ctx, int64_t rows, int64_t cols, const void* Z, int64_t ldz, const void* dF,
                        int64_t lddf, void* dZ, int64_t lddz, plx_dtype dtype) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!dtype_ok(dtype)) return fail(ctx, PLX_ERR_INVALID, "unknown dtype %d", (int)dtype);
    if (rows < 0 || cols < 0) return fail(ctx, PLX_ERR_INVALID, "negative dimension");
    if (rows > 0 && cols > 0 && (!Z || !dF || !dZ)) return fail(ctx, PLX_ERR_INVALID, "Z, dF or dZ is NULL");
    if (ldz < cols || lddf < cols || lddz < cols) return fail(ctx, PLX_ERR_SHAPE, "leading dimension too small");
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");
    if (rows == 0 || cols == 0) return PLX_OK;
    return launch_relu_bwd(ctx, rows, cols, Z, ldz, dF, lddf, dZ, lddz, dtype);
}

plx_status plx_softmax_ce(plx_ctx* ctx, int64_t n, int64_t c, const void* Z, int64_t ldz, const int64_t* y, void* dZ,
                          int64_t lddz, float* row_loss, float* loss, plx_dtype dtype) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!dtype_ok(dtype)) return fail(ctx, PLX_ERR_INVALID, "unknown dtype %d", (int)dtype);
    if (n < 0 || c <= 0) return fail(ctx, PLX_ERR_INVALID, "n must be >= 0 and c > 0");
    if (n > 0 && (!Z || !y || !dZ || !row_loss)) return fail(ctx, PLX_ERR_INVALID, "Z, y, dZ or row_loss is NULL");
    if (ldz < c || lddz < c) return fail(ctx, PLX_ERR_SHAPE, "leading dimension too small");
    if (c > 1024) return fail(ctx, PLX_ERR_UNSUPPORTED, "more than 1024 classes");
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");
    return launch_softmax_ce(ctx, n, c, Z, ldz, y, dZ, lddz, row_loss, loss, dtype);
}

// ---- one GCN layer ------------------------------------------------------------------------------

static plx_order resolve_order(plx_order order, int64_t din, int64_t dout) {
    if (order == PLX_ORDER_AUTO) return din <= dout ? PLX_ORDER_AGG_FIRST : PLX_ORDER_COMBINE_FIRST;
    return order;
}

// Workspace layout (each region 256-byte aligned):
//   COMBINE_FIRST: T / G  [ka x dout]   | dZ [ma x dout] (if act)  | dW partial sums
//   AGG_FIRST    : dS     [ma x din]    | dZ [ma x dout] (if act)  | dW partial sums
// Internal matrices get a leading dimension padded to 16 bytes so every row allows 128-bit accesses; rows shorter
// than 256 bytes get a 64-byte pitch, so that a gathered row never touches a cache line more than it must.
struct LayerWs {
    size_t off_a = 0, off_dz = 0, off_tn = 0, total = 0;
    int64_t ld_in = 0, ld_out = 0;   // padded din / dout in elements
};

static int64_t pad16(int64_t cols, plx_dtype dtype) {
    const int64_t es = (int64_t)elt_size(dtype);
    const int64_t q = (cols * es < 256 ? 64 : 16) / es;
    return (cols + q - 1) / q * q;
}

static LayerWs layer_ws(const Orient& a, int64_t din, int64_t dout, plx_dtype dtype, plx_act act, plx_order order) {
    LayerWs w;
    size_t es = elt_size(dtype);
    w.ld_in = pad16(din, dtype); w.ld_out = pad16(dout, dtype);
    size_t first = order == PLX_ORDER_AGG_FIRST ? (size_t)a.rows * w.ld_in * es : (size_t)a.cols * w.ld_out * es;
    w.off_a = 0;
    w.off_dz = align256(first);
    size_t dz = act != PLX_ACT_NONE ? (size_t)a.rows * w.ld_out * es : 0;
    w.off_tn = w.off_dz + align256(dz);
    int64_t R = order == PLX_ORDER_AGG_FIRST ? a.rows : a.cols;
    w.total = w.off_tn + align256(gemm_tn_workspace(R, din, dout));
    return w;
}

size_t plx_gcn_layer_workspace(const plx_csr* csr, int transposed_A, int64_t din, int64_t dout, plx_dtype dtype,
                               plx_act act, plx_order order) {
    if (!csr || din <= 0 || dout <= 0 || !dtype_ok(dtype)) return 0;
    if ((int)order < 0 || (int)order > 2) return 0;
    return layer_ws(csr->o[transposed_A ? 1 : 0], din, dout, dtype, act, resolve_order(order, din, dout)).total;
}

static plx_status layer_common_checks(plx_ctx* ctx, const plx_csr* csr, int64_t din, int64_t dout, plx_dtype dtype,
                                      plx_act act, plx_order order) {
    if (!csr) return fail(ctx, PLX_ERR_INVALID, "csr is NULL");
    if (!dtype_ok(dtype)) return fail(ctx, PLX_ERR_INVALID, "unknown dtype %d", (int)dtype);
    if (act != PLX_ACT_NONE && act != PLX_ACT_RELU && act != PLX_ACT_RELU_BITS) return fail(ctx, PLX_ERR_INVALID, "unknown activation %d", (int)act);
    if ((int)order < 0 || (int)order > 2) return fail(ctx, PLX_ERR_INVALID, "unknown order %d", (int)order);
    if (din <= 0 || dout <= 0) return fail(ctx, PLX_ERR_INVALID, "din and dout must be positive");
    return PLX_OK;
}

}  // extern "C"

namespace {

// How a forward call departs from plx_gcn_layer_fwd (all zero: it does not).
struct FwdVariant {
    // also Tn[ma x dn] = (this layer's output) Wn, the combine step of the following layer (Wn: dout x dn)
    const float* Wn = nullptr;
    int64_t ldwn = 0, dn = 0;
    void* Tn = nullptr;
    int64_t ldtn = 0;
    // combine-first order with T = H W given by the caller (ka x dout): H and W are not read
    const void* T = nullptr;
    int64_t ldt = 0;
};

plx_status layer_fwd(plx_ctx* ctx, const plx_csr* csr, int transposed_A, const void* H, int64_t ldh,
                     const float* W, int64_t ldw, int64_t din, int64_t dout, plx_dtype dtype, plx_act act,
                     plx_order order, void* Z, int64_t ldz, void* F, int64_t ldf, void* saved,
                     int64_t ldsaved, void* ws, size_t ws_bytes, const FwdVariant& var) {
    if (!ctx) return PLX_ERR_INVALID;
    PLX_TRY(layer_common_checks(ctx, csr, din, dout, dtype, act, order));
    const Orient& a = csr->o[transposed_A ? 1 : 0];
    order = resolve_order(order, din, dout);
    if (a.rows == 0 && a.cols == 0)        // the adjacency of a graph without nodes: no matrix of the layer has a row (pointers may be NULL)
        return ctx->dry ? fail(ctx, PLX_ERR_DEVICE, "validate-only context") : PLX_OK;
    if (var.T) {
        if (var.ldt < dout) return fail(ctx, PLX_ERR_SHAPE, "ldt smaller than dout");
    } else if (!H || !W) {
        return fail(ctx, PLX_ERR_INVALID, "H or W is NULL");
    }
    if (var.Tn) {
        if (!var.Wn || var.dn <= 0) return fail(ctx, PLX_ERR_INVALID, "Wn is NULL or dn is not positive");
        if (var.ldwn < var.dn || var.ldtn < var.dn) return fail(ctx, PLX_ERR_SHAPE, "ldwn or ldtn smaller than dn");
        if (act != PLX_ACT_NONE && !F) return fail(ctx, PLX_ERR_INVALID, "the following layer reads F: it must be given");
    }
    if (!Z && !F) return fail(ctx, PLX_ERR_INVALID, "Z and F are both NULL");
    const bool sign_bits = act == PLX_ACT_RELU_BITS;          // Z receives one bit per element instead of the values
    if (sign_bits && (!Z || !F)) return fail(ctx, PLX_ERR_INVALID, "the sign-bit activation writes both Z (bits) and F");
    if (sign_bits && (reinterpret_cast<uintptr_t>(Z) & 3)) return fail(ctx, PLX_ERR_INVALID, "the sign bits need a 4-byte aligned Z");
    if ((!var.T && (ldh < din || ldw < dout)) || (Z && ldz < (sign_bits ? (dout + 31) / 32 : dout)) || (F && ldf < dout))
        return fail(ctx, PLX_ERR_SHAPE, "leading dimension too small");
    if (order == PLX_ORDER_AGG_FIRST) {
        if (!saved) return fail(ctx, PLX_ERR_INVALID, "aggregate-first order needs the `saved` buffer");
        if (ldsaved < din) return fail(ctx, PLX_ERR_SHAPE, "ldsaved smaller than din");
    }
    LayerWs w = layer_ws(a, din, dout, dtype, act, order);
    if (order == PLX_ORDER_COMBINE_FIRST && !var.T && (!ws || ws_bytes < w.total))
        return fail(ctx, PLX_ERR_SHAPE, "workspace of %zu bytes is smaller than the %zu needed", ws_bytes, w.total);
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");

    if (a.rows == 0) return PLX_OK;          // no output rows
    if (a.cols == 0 || a.nnz == 0) {
        // an adjacency without entries: every output is zero (A H = 0, ReLU(0) = 0, sign bits 0, F Wn = 0)
        const size_t es = elt_size(dtype);
        if (order == PLX_ORDER_AGG_FIRST) PLX_TRY(launch_zero(ctx, a.rows, din, saved, ldsaved, es));
        if (sign_bits) PLX_TRY(launch_zero(ctx, a.rows, (dout + 31) / 32, Z, ldz, sizeof(uint32_t)));
        else PLX_TRY(launch_zero(ctx, a.rows, dout, Z, ldz, es));
        PLX_TRY(launch_zero(ctx, a.rows, dout, F, ldf, es));
        PLX_TRY(launch_zero(ctx, a.rows, var.dn, var.Tn, var.ldtn, es));
        return PLX_OK;
    }
    // The last product of the layer stores the pre-activation (if wanted) and the activated
    // output (Eq. 2.3) from the same registers.
    void* plain = sign_bits ? nullptr : Z;
    void* activated = nullptr;
    uint32_t* bits = sign_bits ? static_cast<uint32_t*>(Z) : nullptr;
    if (F) {
        if (act != PLX_ACT_NONE) activated = F;
        else if (!Z) plain = F;              // no activation and only F wanted: F is the plain output
    }
    const int64_t ld_plain = plain == Z ? ldz : ldf;
    bool next_done = false;                  // Tn written by the product that wrote this layer's output
    if (order == PLX_ORDER_AGG_FIRST && ctx->fused_aggregation && !var.Tn &&
        spmm_combine_supported(a, H, ldh, saved, ldsaved, din, dout, dtype)) {
        // Eq. 2.1, 2.2 and 2.3 in one pass over the adjacency: the aggregated tile is multiplied by W before it leaves the chip
        PLX_TRY(launch_spmm_combine(ctx, a, H, ldh, saved, ldsaved, W, ldw, din, dout, plain, ld_plain, activated, ldf, bits, ldz));
    } else if (order == PLX_ORDER_AGG_FIRST) {
        PLX_TRY(launch_spmm(ctx, a, H, ldh, saved, ldsaved, din, dtype));                    // Eq. 2.1
        if (var.Tn && gemm_next_supported(ctx, a.rows, dout, din, var.dn, dtype, saved, ldsaved, plain ? ld_plain : 0,
                                          activated ? ldf : 0, var.ldtn)) {
            // Eq. 2.2 (+2.3) of this layer and Eq. 2.2 of the next one from the same tile
            PLX_TRY(launch_gemm(ctx, false, a.rows, dout, din, saved, ldsaved, W, ldw, plain, ld_plain, dtype, activated, ldf, bits,
                                ldz, var.Wn, var.ldwn, var.dn, static_cast<float*>(var.Tn), var.ldtn));
            next_done = true;
        } else {
            PLX_TRY(launch_gemm(ctx, false, a.rows, dout, din, saved, ldsaved, W, ldw, plain, ld_plain, dtype, activated, ldf, bits,
                                ldz));                                                       // Eq. 2.2 (+2.3)
        }
    } else {
        const void* T = var.T;
        int64_t ldt = var.ldt;
        if (!T) {
            void* Tw = static_cast<char*>(ws) + w.off_a;
            PLX_TRY(launch_gemm(ctx, false, a.cols, dout, din, H, ldh, W, ldw, Tw, w.ld_out, dtype));
            T = Tw; ldt = w.ld_out;
        }
        PLX_TRY(launch_spmm(ctx, a, T, ldt, plain, ld_plain, dout, dtype, activated, ldf));
        if (bits) PLX_TRY(launch_bits_from_act(ctx, a.rows, dout, F, ldf, bits, ldz, dtype));
    }
    if (F && act == PLX_ACT_NONE && Z && F != Z)
        PLX_HIP(ctx, hipMemcpy2DAsync(F, ldf * elt_size(dtype), Z, ldz * elt_size(dtype), dout * elt_size(dtype), a.rows,
                                      hipMemcpyDeviceToDevice, ctx->stream));
    if (var.Tn && !next_done) {              // elsewhere the following layer's product is a product of its own
        const void* out = act != PLX_ACT_NONE ? F : (plain == Z ? Z : F);
        const int64_t ldout = out == Z ? ldz : ldf;
        PLX_TRY(launch_gemm(ctx, false, a.rows, var.dn, dout, out, ldout, var.Wn, var.ldwn, var.Tn, var.ldtn, dtype));
    }
    return PLX_OK;
}

}  // namespace

extern "C" {

plx_status plx_gcn_layer_fwd(plx_ctx* ctx, const plx_csr* csr, int transposed_A, const void* H, int64_t ldh,
                             const float* W, int64_t ldw, int64_t din, int64_t dout, plx_dtype dtype, plx_act act,
                             plx_order order, void* Z, int64_t ldz, void* F, int64_t ldf, void* saved,
                             int64_t ldsaved, void* ws, size_t ws_bytes) {
    return layer_fwd(ctx, csr, transposed_A, H, ldh, W, ldw, din, dout, dtype, act, order, Z, ldz, F, ldf, saved, ldsaved, ws,
                     ws_bytes, FwdVariant{});
}

plx_status plx_gcn_layer_fwd_chained(plx_ctx* ctx, const plx_csr* csr, int transposed_A, const void* H, int64_t ldh,
                                     const float* W, int64_t ldw, int64_t din, int64_t dout, plx_dtype dtype, plx_act act,
                                     plx_order order, void* Z, int64_t ldz, void* F, int64_t ldf, void* saved,
                                     int64_t ldsaved, const float* Wn, int64_t ldwn, int64_t dn, void* Tn, int64_t ldtn,
                                     void* ws, size_t ws_bytes) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!Tn) return fail(ctx, PLX_ERR_INVALID, "Tn is NULL");
    FwdVariant var;
    var.Wn = Wn; var.ldwn = ldwn; var.dn = dn; var.Tn = Tn; var.ldtn = ldtn;
    return layer_fwd(ctx, csr, transposed_A, H, ldh, W, ldw, din, dout, dtype, act, order, Z, ldz, F, ldf, saved, ldsaved, ws,
                     ws_bytes, var);
}

plx_status plx_gcn_layer_fwd_from_t(plx_ctx* ctx, const plx_csr* csr, int transposed_A, const void* T, int64_t ldt,
                                    int64_t dout, plx_dtype dtype, plx_act act, void* Z, int64_t ldz, void* F, int64_t ldf) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!T) return fail(ctx, PLX_ERR_INVALID, "T is NULL");
    FwdVariant var;
    var.T = T; var.ldt = ldt;
    return layer_fwd(ctx, csr, transposed_A, nullptr, 0, nullptr, 0, dout, dout, dtype, act, PLX_ORDER_COMBINE_FIRST, Z, ldz, F, ldf,
                     nullptr, 0, nullptr, 0, var);
}

}  // extern "C"

namespace {

// How a backward call departs from plx_gcn_layer_bwd (all zero: it does not).
struct BwdVariant {
    // the upstream gradient in factored form, dF = Gn Wn^T (Gn: ma x dn, dtype of the layer; Wn: dout x dn), instead of dF
    const void* Gn = nullptr;
    int64_t ldgn = 0;
    const float* Wn = nullptr;
    int64_t ldwn = 0, dn = 0;
    // combine-first order: A^T dZ goes here instead of into the workspace, and Eq. 2.6 (dH) is left to the caller
    void* dT = nullptr;
    int64_t lddt = 0;
};

// bytes of the formed gradient behind the layer workspace (layer_bwd with factors outside the fused kernel's range)
size_t formed_gradient_bytes(const Orient& a, int64_t dout, plx_dtype dtype) {
    return align256((size_t)a.rows * pad16(dout, dtype) * elt_size(dtype));
}

plx_status layer_bwd(plx_ctx* ctx, const plx_csr* csr, int transposed_A, const void* H, int64_t ldh,
                     const float* W, int64_t ldw, const void* Z, int64_t ldz, const void* dF, int64_t lddf,
                     const void* saved, int64_t ldsaved, int64_t din, int64_t dout, plx_dtype dtype,
                     plx_act act, plx_order order, void* dH, int64_t lddh, float* dW, int64_t lddw, void* ws,
                     size_t ws_bytes, const BwdVariant& var) {
    if (!ctx) return PLX_ERR_INVALID;
    PLX_TRY(layer_common_checks(ctx, csr, din, dout, dtype, act, order));
    const int t = transposed_A ? 1 : 0;
    const Orient& a = csr->o[t];
    const Orient& at = csr->o[1 - t];   // the transpose of the layer's adjacency
    order = resolve_order(order, din, dout);
    if (a.rows == 0 && a.cols == 0) {      // a graph without nodes: only dW exists, and it is zero
        if (!dW || lddw < dout) return fail(ctx, !dW ? PLX_ERR_INVALID : PLX_ERR_SHAPE, "dW is NULL or lddw smaller than dout");
        if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");
        return launch_zero(ctx, din, dout, dW, lddw, sizeof(float));
    }
    if (var.dT) {
        if (order != PLX_ORDER_COMBINE_FIRST) return fail(ctx, PLX_ERR_INVALID, "the gradient of H W exists only in combine-first order");
        if (var.lddt < dout) return fail(ctx, PLX_ERR_SHAPE, "lddt smaller than dout");
        if (dH) return fail(ctx, PLX_ERR_INTERNAL, "dT and dH are alternatives");
    } else if (!W) {
        return fail(ctx, PLX_ERR_INVALID, "W is NULL");
    }
    if (var.Gn) {
        if (!var.Wn || var.dn <= 0) return fail(ctx, PLX_ERR_INVALID, "Wn is NULL or dn is not positive");
        if (var.ldgn < var.dn || var.ldwn < var.dn) return fail(ctx, PLX_ERR_SHAPE, "leading dimension of a factor smaller than dn");
        lddf = dout;          // dF is formed here: its own leading dimension is not the caller's
    }
    if ((!dF && !var.Gn) || !dW) return fail(ctx, PLX_ERR_INVALID, "dF or dW is NULL");
    const bool sign_bits = act == PLX_ACT_RELU_BITS;
    if (act != PLX_ACT_NONE && !Z) return fail(ctx, PLX_ERR_INVALID, "Z is needed for the ReLU derivative");
    if (sign_bits && (reinterpret_cast<uintptr_t>(Z) & 3)) return fail(ctx, PLX_ERR_INVALID, "the sign bits need a 4-byte aligned Z");
    if (ldw < dout || lddf < dout || lddw < dout || (Z && ldz < (sign_bits ? (dout + 31) / 32 : dout)) ||
        (dH && lddh < din))
        return fail(ctx, PLX_ERR_SHAPE, "leading dimension too small");
    if (order == PLX_ORDER_AGG_FIRST) {
        if (!saved) return fail(ctx, PLX_ERR_INVALID, "aggregate-first order needs the `saved` buffer");
        if (ldsaved < din) return fail(ctx, PLX_ERR_SHAPE, "ldsaved smaller than din");
    } else {
        if (!H) return fail(ctx, PLX_ERR_INVALID, "H is NULL");
        if (ldh < din) return fail(ctx, PLX_ERR_SHAPE, "ldh smaller than din");
    }
    LayerWs w = layer_ws(a, din, dout, dtype, act, order);
    const void* mask = act != PLX_ACT_NONE ? Z : nullptr;
    // the fused kernels address a tile with 31-bit byte offsets; wider leading dimensions take the separate products
    const int64_t ld_max = std::max(std::max(std::max(ldsaved, ldh), std::max(std::max(lddf, ldz), lddh)), std::max(var.lddt, var.ldgn));
    const bool fused = bwd_dense_supported(din, dout, dtype) && (ld_max < (int64_t(1) << 23) || dtype == PLX_BF16);
    // factors: does the fused kernel form dF itself, or is it formed once behind the layer workspace?
    const bool in_kernel = var.Gn && fused && order == PLX_ORDER_AGG_FIRST &&
                           bwd_dense_factor_supported(ctx, a.rows, din, dout, var.dn, dtype, saved, ldsaved, var.Gn, var.ldgn, ldz,
                                                      w.ld_in, mask && !sign_bits);
    const size_t need = w.total + ((var.Gn && !in_kernel) ? formed_gradient_bytes(a, dout, dtype) : 0);
    if (!ws || ws_bytes < need)
        return fail(ctx, PLX_ERR_SHAPE, "workspace of %zu bytes is smaller than the %zu needed", ws_bytes, need);
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");

    if (a.nnz == 0) {
        // an adjacency without entries (or without rows or columns): A H = 0 and A^T dZ = 0, so every gradient is zero
        PLX_TRY(launch_zero(ctx, din, dout, dW, lddw, sizeof(float)));
        PLX_TRY(launch_zero(ctx, a.cols, din, dH, lddh, elt_size(dtype)));
        PLX_TRY(launch_zero(ctx, a.cols, dout, var.dT, var.lddt, elt_size(dtype)));
        return PLX_OK;
    }
    char* base = static_cast<char*>(ws);
    void* tn_ws = base + w.off_tn;
    size_t tn_bytes = w.total - w.off_tn;
    if (var.Gn) {
        if (in_kernel) {
            // Eq. 2.6 of the following layer, then Eq. 2.4 + 2.5 + 2.6 of this one, tile by tile: dF never exists in memory
            void* dS = dH ? base + w.off_a : nullptr;
            PLX_TRY(launch_bwd_dense(ctx, a.rows, din, dout, saved, ldsaved, nullptr, 0, mask, ldz, W, ldw, dS, w.ld_in, dW, lddw,
                                     dtype, tn_ws, tn_bytes, sign_bits, static_cast<const float*>(var.Gn), var.ldgn, var.Wn, var.ldwn,
                                     var.dn));
            if (dH) PLX_TRY(launch_spmm(ctx, at, dS, w.ld_in, dH, lddh, din, dtype));        // Eq. 2.7
            return PLX_OK;
        }
        // elsewhere the product is formed once, behind the layer workspace, and the call goes on as with a given dF
        void* formed = base + w.total;
        PLX_TRY(launch_gemm(ctx, true, a.rows, dout, var.dn, var.Gn, var.ldgn, var.Wn, var.ldwn, formed, w.ld_out, dtype));
        dF = formed;
        lddf = w.ld_out;
    }
    if (fused) {
        // Eq. 2.4 is applied while the gradient tile is loaded; it is never written back
        if (order == PLX_ORDER_AGG_FIRST) {
            void* dS = dH ? base + w.off_a : nullptr;
            PLX_TRY(launch_bwd_dense(ctx, a.rows, din, dout, saved, ldsaved, dF, lddf, mask, ldz, W, ldw, dS, w.ld_in, dW, lddw,
                                     dtype, tn_ws, tn_bytes, sign_bits));                    // Eq. 2.4 + 2.5 + 2.6
            if (dH) PLX_TRY(launch_spmm(ctx, at, dS, w.ld_in, dH, lddh, din, dtype));        // Eq. 2.7
        } else {
            const void* dZ = dF;
            int64_t lddz = lddf;
            if (mask) {
                void* buf = base + w.off_dz;
                PLX_TRY(launch_relu_bwd(ctx, a.rows, dout, Z, ldz, dF, lddf, buf, w.ld_out, dtype, sign_bits));
                dZ = buf; lddz = w.ld_out;
            }
            void* G = var.dT ? var.dT : base + w.off_a;
            const int64_t ldg = var.dT ? var.lddt : w.ld_out;
            PLX_TRY(launch_spmm(ctx, at, dZ, lddz, G, ldg, dout, dtype));                    // A^T dZ
            PLX_TRY(launch_bwd_dense(ctx, a.cols, din, dout, H, ldh, G, ldg, nullptr, 0, W, ldw, dH, lddh, dW, lddw, dtype,
                                     tn_ws, tn_bytes));
        }
        return PLX_OK;
    }
    const void* dZ = dF;
    int64_t lddz = lddf;
    if (mask) {                                                                              // Eq. 2.4
        void* buf = base + w.off_dz;
        PLX_TRY(launch_relu_bwd(ctx, a.rows, dout, Z, ldz, dF, lddf, buf, w.ld_out, dtype, sign_bits));
        dZ = buf; lddz = w.ld_out;
    }
    if (order == PLX_ORDER_AGG_FIRST) {
        PLX_TRY(launch_gemm_tn(ctx, a.rows, din, dout, saved, ldsaved, dZ, lddz, dW, lddw, dtype, tn_ws, tn_bytes));  // Eq. 2.5
        if (dH) {
            void* dS = base + w.off_a;
            PLX_TRY(launch_gemm(ctx, true, a.rows, din, dout, dZ, lddz, W, ldw, dS, w.ld_in, dtype));  // Eq. 2.6
            PLX_TRY(launch_spmm(ctx, at, dS, w.ld_in, dH, lddh, din, dtype));                // Eq. 2.7
        }
    } else {
        void* G = var.dT ? var.dT : base + w.off_a;
        const int64_t ldg = var.dT ? var.lddt : w.ld_out;
        PLX_TRY(launch_spmm(ctx, at, dZ, lddz, G, ldg, dout, dtype));                        // A^T dZ
        PLX_TRY(launch_gemm_tn(ctx, a.cols, din, dout, H, ldh, G, ldg, dW, lddw, dtype, tn_ws, tn_bytes));
        if (dH) PLX_TRY(launch_gemm(ctx, true, a.cols, din, dout, G, ldg, W, ldw, dH, lddh, dtype));
    }
    return PLX_OK;
}

}  // namespace

extern "C" {

plx_status plx_gcn_layer_bwd(plx_ctx* ctx, const plx_csr* csr, int transposed_A, const void* H, int64_t ldh,
                             const float* W, int64_t ldw, const void* Z, int64_t ldz, const void* dF, int64_t lddf,
                             const void* saved, int64_t ldsaved, int64_t din, int64_t dout, plx_dtype dtype,
                             plx_act act, plx_order order, void* dH, int64_t lddh, float* dW, int64_t lddw, void* ws,
                             size_t ws_bytes) {
    return layer_bwd(ctx, csr, transposed_A, H, ldh, W, ldw, Z, ldz, dF, lddf, saved, ldsaved, din, dout, dtype, act, order, dH,
                     lddh, dW, lddw, ws, ws_bytes, BwdVariant{});
}

plx_status plx_gcn_layer_bwd_dt(plx_ctx* ctx, const plx_csr* csr, int transposed_A, const void* H, int64_t ldh,
                                const void* Z, int64_t ldz, const void* dF, int64_t lddf, int64_t din, int64_t dout,
                                plx_dtype dtype, plx_act act, void* dT, int64_t lddt, float* dW, int64_t lddw, void* ws,
                                size_t ws_bytes) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!dT) return fail(ctx, PLX_ERR_INVALID, "dT is NULL");
    BwdVariant var;
    var.dT = dT; var.lddt = lddt;
    return layer_bwd(ctx, csr, transposed_A, H, ldh, nullptr, dout, Z, ldz, dF, lddf, nullptr, 0, din, dout, dtype, act,
                     PLX_ORDER_COMBINE_FIRST, nullptr, 0, dW, lddw, ws, ws_bytes, var);
}

plx_status plx_gcn_layer_plan(const plx_ctx* ctx, int64_t din, int64_t dout, int64_t dn, plx_dtype dtype, plx_order order,
                              plx_order next_order, int keep_values, int* agg_first, int* sign_bits, int* chain_fwd,
                              int* chain_bwd) {
    if (!ctx) return PLX_ERR_INVALID;
    if (din <= 0 || dout <= 0 || dn < 0 || !dtype_ok(dtype) || (int)order < 0 || (int)order > 2 || (int)next_order < 0 ||
        (int)next_order > 2)
        return PLX_ERR_INVALID;
    const bool agg = resolve_order(order, din, dout) == PLX_ORDER_AGG_FIRST;
    // the dense kernels of an aggregate-first layer of widths up to 128 pack the sign of their result while they write it
    const bool bits = !keep_values && agg && din <= 128 && dout <= 128;
    // a following combine-first layer starts with a product over this layer's output rows and ends with one: both can
    // run inside this layer's dense kernels (16-byte aligned rows are the caller's to provide: the calls fall back to
    // separate products otherwise).  One 16-column step of dn only: wider factors were measured slower than the matrix
    // they avoid.
    const bool pair = dn > 0 && dn <= 16 && agg && resolve_order(next_order, dout, dn) == PLX_ORDER_COMBINE_FIRST;
    const int64_t ld4 = 4;
    if (agg_first) *agg_first = agg;
    if (sign_bits) *sign_bits = bits;
    if (chain_fwd) *chain_fwd = pair && gemm_next_supported(ctx, 1, dout, din, dn, dtype, nullptr, ld4, ld4, ld4, ld4);
    if (chain_bwd) *chain_bwd = pair && bwd_dense_supported(din, dout, dtype) &&
                                bwd_dense_factor_supported(ctx, 1, din, dout, dn, dtype, nullptr, ld4, nullptr, ld4, 0, 0,
                                                           /*value_mask=*/keep_values != 0);
    return PLX_OK;
}

size_t plx_gcn_layer_bwd_chained_workspace(const plx_ctx* ctx, const plx_csr* csr, int transposed_A, int64_t din, int64_t dout,
                                           int64_t dn, plx_dtype dtype, plx_act act, plx_order order) {
    const size_t base = plx_gcn_layer_workspace(csr, transposed_A, din, dout, dtype, act, order);
    if (base == 0 || !ctx || dn <= 0) return 0;
    const Orient& a = csr->o[transposed_A ? 1 : 0];
    // with 16-byte aligned rows (checked with the pointers, at the call) these shapes never form dF in memory
    const int64_t ld4 = 4;
    const bool in_kernel = resolve_order(order, din, dout) == PLX_ORDER_AGG_FIRST && act != PLX_ACT_RELU &&
                           bwd_dense_factor_supported(ctx, a.rows, din, dout, dn, dtype, nullptr, ld4, nullptr, ld4, 0, 0, false);
    return base + (in_kernel ? 0 : formed_gradient_bytes(a, dout, dtype));
}

plx_status plx_gcn_layer_bwd_chained(plx_ctx* ctx, const plx_csr* csr, int transposed_A, const void* H, int64_t ldh,
                                     const float* W, int64_t ldw, const void* Z, int64_t ldz, const void* dTn, int64_t lddtn,
                                     const float* Wn, int64_t ldwn, int64_t dn, const void* saved, int64_t ldsaved,
                                     int64_t din, int64_t dout, plx_dtype dtype, plx_act act, plx_order order, void* dH,
                                     int64_t lddh, float* dW, int64_t lddw, void* ws, size_t ws_bytes) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!csr) return fail(ctx, PLX_ERR_INVALID, "csr is NULL");
    if (!dTn) return fail(ctx, PLX_ERR_INVALID, "dTn is NULL");
    if (!dtype_ok(dtype) || dout <= 0) return fail(ctx, PLX_ERR_INVALID, "unknown dtype or dout not positive");
    BwdVariant var;
    var.Gn = dTn; var.ldgn = lddtn; var.Wn = Wn; var.ldwn = ldwn; var.dn = dn;
    return layer_bwd(ctx, csr, transposed_A, H, ldh, W, ldw, Z, ldz, nullptr, 0, saved, ldsaved, din, dout, dtype, act, order, dH,
                     lddh, dW, lddw, ws, ws_bytes, var);
}

}  // extern "C"
