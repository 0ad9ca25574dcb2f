// Internal declarations shared by the library's translation units (not installed).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <string>
#include <vector>

#include "plx.h"

namespace plx {

constexpr int kWave = 64;            // gfx950 wavefront width
constexpr int kNumClasses = 34;      // row-length classes: 0 = empty, c = 1 + floor(log2 len)
constexpr int kSubwaveMaxClass = 8;  // rows shorter than 2^8 are handled by a group of lanes
constexpr int kLongClass = 13;       // without column windows only rows with len >= 2^12 are split into segments
constexpr int64_t kSegLen = 2048;    // most nonzeros a segment may hold
constexpr int kPartFloats = 128;     // partial-sum floats a handle keeps per segment: the widest pass of the segment kernels

// One stored orientation of the adjacency (CSR) plus its row binning.
struct Orient {
    int64_t rows = 0, cols = 0, nnz = 0;
    int64_t* rowptr = nullptr;     // device [rows + 1], canonical row pointers (row id order)
    // Entries are STORED IN BINNED ORDER: slot s of row_order holds row row_order[s], whose entries
    // (columns strictly ascending) are col/val[bptr[s] .. bptr[s+1]).  Rows of one length class are
    // therefore contiguous in memory and the kernels stream the CSR arrays.
    int32_t* col = nullptr;        // device [nnz]
    float* val = nullptr;          // device [nnz]
    int32_t* bptr = nullptr;       // device [rows + 1]: slot pointers into col/val
    int32_t* row_order = nullptr;  // device [rows]: row ids sorted by (row block, length class), ascending id inside
    // Row blocks (blocked aggregation, paper Sec. 5.2): block b holds rows [b*rows_per_block, ...).  The
    // slot list is sorted by block first, so every block owns one contiguous slot range per class.
    int n_blocks = 1;
    int64_t rows_per_block = 0;
    std::vector<int64_t> boff;     // host [n_blocks * (kNumClasses + 1)]: first slot of class c in block b
    std::vector<int64_t> bnnz;     // host [n_blocks * kNumClasses]: stored entries per (block, class)
    std::vector<int64_t> long0;    // host [n_blocks + 1]: first long row (index into long_row) of block b
    std::vector<int64_t> seg0b;    // host [n_blocks + 1]: first segment of block b
    int64_t off(int b, int c) const { return boff[(size_t)b * (kNumClasses + 1) + c]; }
    int tag = 0;                               // 0 = forward orientation, 1 = its transpose (timing labels)
    // Rows of class >= long_class are cut into segments: at the boundaries of n_windows equal column
    // windows, and to at most seg_max nonzeros.  Segments are numbered row by row (the order their
    // partial sums are added in) and launched window by window (seg_launch), so that the wavefronts
    // running at any moment gather from a narrow band of the dense operand that stays in cache.
    int n_windows = 1, long_class = kLongClass;
    int32_t seg_max = (int32_t)kSegLen;
    int32_t* seg_launch = nullptr; // device [n_seg] segment ids in launch order (block, window, row)
    int64_t n_long = 0, n_seg = 0;
    int32_t* long_row = nullptr;   // device [n_long] row id
    int32_t* long_seg0 = nullptr;  // device [n_long + 1] first segment of each long row
    int64_t* seg_lo = nullptr;     // device [n_seg] first entry of the segment (binned storage)
    int32_t* seg_len = nullptr;    // device [n_seg] nonzeros in the segment
    int4* seg_desc = nullptr;      // device [n_seg], launch order: {first entry, nonzeros, segment id, 0} -- what a wavefront of
                                   // the segment kernel needs, in one 16-byte load at a wave-uniform address
    float* part = nullptr;         // device [n_seg * kPartFloats] partial sums of the segments (sized with the handle, so that
                                   // a product allocates nothing and never waits)
};

}  // namespace plx

struct plx_ctx {
    int device = -1;
    bool dry = false;  // validate-only context
    hipStream_t stream = nullptr;
    int n_cu = 256;    // compute units of the device
    plx_alloc_fn alloc = nullptr;
    plx_free_fn release = nullptr;
    void* user = nullptr;
    std::string err;
    int n_windows = 8;        // column windows for the rows handled through segments (1 = none); measured optimum 4-12
    bool split_products = true;   // fp32 dense products of the wide layers through six bf16 matrix instructions
    bool fused_aggregation = false;   // aggregate-first forward: Eq. 2.2-2.3 in the epilogue of the sparse kernels (measured slower)
    // optional per-kernel timing (plx_timing_enable)
    struct Timed { std::string name; hipEvent_t start, stop; };
    bool timing = false;
    std::vector<Timed> timed;
};

struct plx_csr {
    plx::Orient o[2];        // [0] = A_fwd, [1] = A_fwd^T
    int64_t n_deg = 0;
    int64_t* deg = nullptr;  // device [n_deg], original id order (handles from plx_build_csr only)
};

namespace plx {

plx_status fail(plx_ctx* ctx, plx_status s, const char* fmt, ...);
void* dev_alloc(plx_ctx* ctx, size_t bytes);   // NULL on failure (error recorded)
void dev_free(plx_ctx* ctx, void* p);

#define PLX_HIP(ctx, call)                                                                   \
    do {                                                                                     \
        hipError_t e_ = (call);                                                              \
        if (e_ != hipSuccess)                                                                \
            return plx::fail((ctx), PLX_ERR_DEVICE, "%s failed: %s", #call, hipGetErrorString(e_)); \
    } while (0)

#define PLX_TRY(expr)                    \
    do {                                 \
        plx_status s_ = (expr);          \
        if (s_ != PLX_OK) return s_;     \
    } while (0)

// RAII holder for temporaries obtained through the context allocator.
struct TempPool {
    plx_ctx* ctx;
    std::vector<void*> ptrs;
    explicit TempPool(plx_ctx* c) : ctx(c) {}
    ~TempPool() { for (void* p : ptrs) dev_free(ctx, p); }
    template <typename T> T* get(size_t count) {
        void* p = dev_alloc(ctx, (count ? count : 1) * sizeof(T));
        if (p) ptrs.push_back(p);
        return static_cast<T*>(p);
    }
};

// Brackets the kernel launches made during its lifetime with two events when timing is on.
struct KernelTimer {
    plx_ctx* ctx;
    bool on;
    plx_ctx::Timed t;
    KernelTimer(plx_ctx* c, const std::string& name, bool allowed = true) : ctx(c), on(c->timing && allowed) {
        if (!on) return;
        t.name = name;
        if (hipEventCreate(&t.start) != hipSuccess || hipEventCreate(&t.stop) != hipSuccess) { on = false; return; }
        (void)hipEventRecord(t.start, ctx->stream);
    }
    ~KernelTimer() {
        if (!on) return;
        (void)hipEventRecord(t.stop, ctx->stream);
        ctx->timed.push_back(t);
    }
};

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// set-up: fills the binning fields of `o` from its canonical CSR arrays and re-orders the entries
// into binned storage (waits on the stream)
plx_status build_bins(plx_ctx* ctx, Orient& o, int n_blocks = 1);
// column windows / segment length used by build_bins for an orientation with the given shape
void segment_policy(const plx_ctx* ctx, int64_t rows, int64_t cols, int64_t nnz, int* n_windows, int* long_class, int32_t* seg_max);
// undoes build_bins: entries back in canonical CSR order, binning fields released
plx_status unbin(plx_ctx* ctx, Orient& o);
// copies the entries of `o` back into canonical CSR order (either output may be NULL)
plx_status export_entries(plx_ctx* ctx, const Orient& o, int32_t* col, float* val);
void free_orient(plx_ctx* ctx, Orient& o);

// kernels' host launchers (all asynchronous on ctx->stream)
// Y = A X (Y may be NULL); if Yact != NULL it also receives max(A X, 0).  block >= 0 restricts the
// product to the rows of that row block (other rows of Y are not touched)
plx_status launch_spmm(plx_ctx* ctx, const Orient& o, const void* X, int64_t ldx, void* Y, int64_t ldy,
                       int64_t d, plx_dtype dtype, void* Yact = nullptr, int64_t ldyact = 0, int block = -1,
                       float* partials = nullptr, size_t partials_bytes = 0);
// Eq. 2.1 with Eq. 2.2 (+ 2.3) in its epilogue: S = A X is written, and C = S W, Fact = max(S W, 0), sign bits as wanted
bool spmm_combine_supported(const Orient& o, const void* X, int64_t ldx, const void* S, int64_t lds_, int64_t din, int64_t dout,
                            plx_dtype dtype);
plx_status launch_spmm_combine(plx_ctx* ctx, const Orient& o, const void* X, int64_t ldx, void* S, int64_t lds_, const float* W,
                               int64_t ldw, int64_t din, int64_t dout, void* C, int64_t ldc, void* Fact, int64_t ldf, uint32_t* bits,
                               int64_t ldbits);
// partials != NULL: the partial sums of split rows go there instead of into the context's buffer; the call then
// allocates nothing, records no timing events, and fails with PLX_ERR_UNSUPPORTED if partials_bytes is too small.
// The fixed per-GPU buffer of plx_spmm_static (resolved once per device, with that device current; NULL on failure):
float* static_partials(plx_ctx* ctx, size_t* bytes);
// C = A op(B) (C may be NULL); if Fact != NULL it also receives max(C, 0); if bits != NULL it receives
// the sign bits [C > 0] (bit j % 32 of word j / 32 of row i, ldbits words per row)
plx_status launch_gemm(plx_ctx* ctx, bool bt, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                       const float* B, int64_t ldb, void* C, int64_t ldc, plx_dtype dtype, void* Fact = nullptr,
                       int64_t ldf = 0, uint32_t* bits = nullptr, int64_t ldbits = 0, const float* Wn = nullptr, int64_t ldwn = 0,
                       int64_t dn = 0, float* Tn = nullptr, int64_t ldtn = 0);
// Tn != NULL: the nn product also writes Tn[M x dn] = act(A B) Wn (Wn: N x dn); only where this holds:
bool gemm_next_supported(const plx_ctx* ctx, int64_t M, int64_t N, int64_t K, int64_t dn, plx_dtype dtype, const void* A, int64_t lda,
                         int64_t ldc, int64_t ldf, int64_t ldtn);
// bits[i][j] = [F[i][j] > 0] for an activated matrix F (used where no producing kernel writes the bits itself)
plx_status launch_bits_from_act(plx_ctx* ctx, int64_t rows, int64_t cols, const void* F, int64_t ldf, uint32_t* bits,
                                int64_t ldbits, plx_dtype dtype);
size_t gemm_tn_workspace(int64_t R, int64_t M, int64_t N);
int64_t tn_rows_per_chunk(int64_t R, int64_t M, int64_t N);
int tn_kslices(int64_t M, int64_t N);
plx_status reduce_partials(plx_ctx* ctx, float* part, int64_t chunks, int64_t M, int64_t N, float* C, int64_t ldc);
// fused Eq. 2.4 + 2.5 + 2.6: dOut = (Q*[Zm>0]) W^T (dOut may be NULL), dW = P^T (Q*[Zm>0]); Zm may be NULL.
// mask_bits: Zm is not a matrix of values but the sign bits written by a forward product (ldz in words)
bool bwd_dense_supported(int64_t Mp, int64_t N, plx_dtype dtype);
plx_status launch_bwd_dense(plx_ctx* ctx, int64_t R, int64_t Mp, int64_t N, const void* P, int64_t ldp, const void* Q,
                            int64_t ldq, const void* Zm, int64_t ldz, const float* W, int64_t ldw, void* dOut, int64_t ldo,
                            float* dW, int64_t lddw, plx_dtype dtype, void* ws, size_t ws_bytes, bool mask_bits = false,
                            const float* G = nullptr, int64_t ldg = 0, const float* Wn = nullptr, int64_t ldwn = 0, int64_t dn = 0);
// G != NULL: Q is not given but formed tile by tile as G[R x dn] Wn[N x dn]^T; only where this holds:
bool bwd_dense_factor_supported(const plx_ctx* ctx, int64_t R, int64_t Mp, int64_t N, int64_t dn, plx_dtype dtype, const void* P,
                                int64_t ldp, const void* G, int64_t ldg, int64_t ldz, int64_t ldo, bool value_mask);
plx_status launch_gemm_tn(plx_ctx* ctx, int64_t R, int64_t M, int64_t N, const void* A, int64_t lda,
                          const void* B, int64_t ldb, float* C, int64_t ldc, plx_dtype dtype, void* ws, size_t ws_bytes);
// rows x cols elements of elt_bytes each set to zero by a kernel (p may be NULL: nothing happens)
plx_status launch_zero(plx_ctx* ctx, int64_t rows, int64_t cols, void* p, int64_t ld, size_t elt_bytes);
plx_status launch_relu(plx_ctx* ctx, int64_t rows, int64_t cols, const void* Z, int64_t ldz, void* F, int64_t ldf,
                       plx_dtype dtype);
plx_status launch_relu_bwd(plx_ctx* ctx, int64_t rows, int64_t cols, const void* Z, int64_t ldz, const void* dF,
                           int64_t lddf, void* dZ, int64_t lddz, plx_dtype dtype, bool mask_bits = false);
plx_status launch_softmax_ce(plx_ctx* ctx, int64_t n, int64_t c, const void* Z, int64_t ldz, const int64_t* y,
                             void* dZ, int64_t lddz, float* row_loss, float* loss, plx_dtype dtype);

// bf16 storage / fp32 accumulation variants (widths up to 128)
plx_status launch_gemm_small_bf16(plx_ctx* ctx, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                                  const float* W, int64_t ldw, void* C, int64_t ldc, void* Fact, int64_t ldf,
                                  uint32_t* bits = nullptr, int64_t ldbits = 0);
plx_status launch_bwd_dense_bf16(plx_ctx* ctx, int64_t R, int64_t Mp, int64_t N, const void* P, int64_t ldp, const void* Q,
                                 int64_t ldq, const void* Zm, int64_t ldz, const float* W, int64_t ldw, void* dOut,
                                 int64_t ldo, float* dW, int64_t lddw, void* ws, size_t ws_bytes, bool mask_bits = false);

inline size_t elt_size(plx_dtype t) { return t == PLX_BF16 ? 2 : 4; }
inline size_t align256(size_t b) { return (b + 255) & ~size_t(255); }

}  // namespace plx
