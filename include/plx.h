/*
 * plx -- the per-GPU hot path of full-graph GCN training with a double-permuted adjacency,
 * for one AMD MI355X (gfx950).  C ABI: plain pointers and sizes only.
 *
 * What a layer computes (paper Sec. 2.1): with A^ = D^-1/2 (A + I) D^-1/2,
 *     aggregation   H = A^ F          (Eq. 2.1, sparse x dense)
 *     combination   Q = H W           (Eq. 2.2, dense x dense)
 *     activation    F' = ReLU(Q)      (Eq. 2.3)
 * and backward (Eq. 2.4-2.7)
 *     dQ = dF' * [Q > 0],  dW = H^T dQ,  dH = dQ W^T,  dF = A^^T dH.
 * The stored adjacency is the double-permuted P_r A^ P_c^T (even layers) and its transpose
 * P_c A^ P_r^T (odd layers), Sec. 5.1, Eq. 5.3-5.4.
 *
 * Pointer kinds.  Every pointer named "device" is memory of the context's GPU; the library
 * never copies it to the host.  `plx_ctx**`, `plx_csr**`, the int64 outputs of plx_csr_dims /
 * plx_csr_bins and strings are host memory.  Dense matrices are row-major with a leading
 * dimension `ld*` counted in ELEMENTS (>= the number of columns).  For PLX_F32 an element is
 * an IEEE fp32; for PLX_BF16 it is a bfloat16 (upper 16 bits of an fp32, round-to-nearest-
 * even on store); sums are always carried in fp32.
 *
 * Ownership.  The caller owns every dense buffer and workspace it passes.  The library owns
 * what is inside a plx_csr (obtained through the context's allocator) until plx_csr_destroy.
 *
 * Execution.  All work is queued on the context's HIP stream and returns without waiting and
 * without allocating device memory (what a product needs beyond its operands is part of the
 * handle or of the caller's workspace), except plx_build_csr, plx_csr_import, plx_csr_export and
 * plx_csr_set_row_blocks, which allocate and wait for their own work (they are set-up calls).  Calls on one context must not overlap in time.
 *
 * Errors.  Every entry point returns a plx_status; nothing aborts or throws across the
 * ABI.  Arguments are checked on the host before any GPU call (NULL, negative sizes,
 * ld < columns, unknown enum, shapes that disagree with the handle), so a bad call leaves
 * the GPU untouched.  plx_last_error gives a one-line description of the last failure on
 * that context.
 */
#ifndef PLX_H
#define PLX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PLX_API __attribute__((visibility("default")))

typedef struct plx_ctx plx_ctx;
typedef struct plx_csr plx_csr;

typedef enum {
    PLX_OK = 0,
    PLX_ERR_INVALID = 1,      /* NULL pointer, negative size, bad enum, bad node id or permutation */
    PLX_ERR_SHAPE = 2,        /* ld < columns, dimensions that disagree with the handle, workspace too small */
    PLX_ERR_UNSUPPORTED = 3,  /* a size or dtype this build does not handle */
    PLX_ERR_OOM = 4,          /* the allocator returned NULL */
    PLX_ERR_DEVICE = 5,       /* no usable GPU, or a HIP call failed */
    PLX_ERR_INTERNAL = 6
} plx_status;

typedef enum { PLX_F32 = 0, PLX_BF16 = 1 } plx_dtype;
typedef enum { PLX_ACT_NONE = 0, PLX_ACT_RELU = 1, PLX_ACT_RELU_BITS = 2 } plx_act;
typedef enum {
    PLX_ORDER_COMBINE_FIRST = 0, /* Z = A^ (H W): the sparse product runs at the output width    */
    PLX_ORDER_AGG_FIRST = 1,     /* Z = (A^ H) W: the order of Eq. 2.1 -> 2.2                      */
    PLX_ORDER_AUTO = 2           /* whichever runs the sparse product at min(d_in, d_out); AGG_FIRST on a tie */
} plx_order;

/* Device-memory allocator hooks (e.g. bound to a framework's caching allocator).  `alloc`
 * returns device memory aligned to at least 256 bytes, or NULL.  Both NULL = hipMalloc/hipFree. */
typedef void* (*plx_alloc_fn)(size_t bytes, void* user);
typedef void (*plx_free_fn)(void* ptr, void* user);

/* ---- context ------------------------------------------------------------------------------
 * device >= 0: a GPU ordinal; hip_stream: a hipStream_t on that device (NULL = the default
 * stream).  device == -1 creates a validate-only context: every entry point still checks its
 * arguments and then returns PLX_ERR_DEVICE instead of touching a GPU (used to test error
 * handling on a machine without one).  Returns PLX_ERR_DEVICE if the GPU cannot be used. */
PLX_API plx_status plx_ctx_create(int device, void* hip_stream, plx_alloc_fn alloc, plx_free_fn release,
                                  void* user, plx_ctx** out);
PLX_API void plx_ctx_destroy(plx_ctx* ctx);
PLX_API const char* plx_last_error(const plx_ctx* ctx);   /* host string owned by the context */
PLX_API const char* plx_status_string(plx_status s);
/* Column windows (a tuning knob; the default of 8 needs no call).  Rows of 256 entries and more
 * are processed as segments cut at the boundaries of n_windows equal column ranges and launched
 * window by window, so that the wavefronts running at any moment gather from a band of the dense
 * operand that stays in the Infinity Cache / L2 instead of coming from HBM each time; the partial
 * sums of a row are added in a fixed order (bit-reproducible).  1 switches the windows off (then
 * only rows of 4096 entries and more are split).  Applies to handles built or re-blocked AFTER the
 * call.  1 <= n_windows <= 64, else PLX_ERR_INVALID. */
PLX_API plx_status plx_ctx_set_column_windows(plx_ctx* ctx, int n_windows);
/* fp32 dense products whose two small dimensions are both 64 or more are bound by the fp32 matrix
 * pipe.  By default (on != 0) they are computed through the bf16 matrix instructions instead: every
 * fp32 operand is the exact sum of three bf16 numbers, and six of the nine bf16 products (all terms
 * down to 2^-23 of the product, i.e. fp32 rounding) are accumulated in fp32, 2.7 times faster than
 * the fp32 instructions.  For finite inputs of any magnitude the results agree with the plain fp32 path
 * to fp32 rounding, but not bit for bit.  An infinite or NaN input makes every result that depends on it
 * NaN (the fp32 instructions give +-infinity where no opposite infinity or zero factor meets it): the
 * same results are non-finite in both paths.  on == 0 selects the plain fp32 instructions everywhere. */
PLX_API plx_status plx_ctx_set_split_products(plx_ctx* ctx, int on);
/* Aggregate-first layers (Eq. 2.1 then 2.2) normally run the sparse product and the dense product as separate kernels, the
 * aggregation H = A F making a round trip through memory between them.  With on != 0, plx_gcn_layer_fwd keeps the
 * aggregated rows on chip and multiplies them by W in the epilogue of the sparse kernels (H is still written once: the
 * backward pass reads it), for fp32 layers with 16 < din <= 32, dout <= 128 and 16-byte aligned rows; other layers are not
 * affected.  Results agree with the separate kernels to fp32 rounding.  Off by default: on the 7M x 28M shard layer the
 * fused kernels were measured slower (the matrix-core epilogue takes registers and LDS from a kernel whose speed is the
 * number of gathers in flight) than the 0.9 GB re-read they save. */
PLX_API plx_status plx_ctx_set_fused_aggregation(plx_ctx* ctx, int on);
PLX_API plx_status plx_sync(plx_ctx* ctx);                /* wait for the context's stream */

/* Optional per-kernel timing for benchmarks.  While enabled, every kernel the library
 * launches is bracketed by two HIP events on the context's stream (a few microseconds of
 * host work per launch, nothing on the GPU).  plx_timing_report waits for the stream, writes
 * one line per kernel name -- "<name> <launches> <total_ms>\n", NUL-terminated, truncated to
 * buf_bytes -- into the HOST buffer `buf`, and clears the record. */
PLX_API plx_status plx_timing_enable(plx_ctx* ctx, int on);
PLX_API plx_status plx_timing_report(plx_ctx* ctx, char* buf, size_t buf_bytes);
/* The same record unaggregated: one line per timed launch, in launch order, "<name> <ms>\n" (a benchmark
 * uses the order to match the launches of a step with a profiler's dispatch list).  Waits for the stream
 * and clears the record like plx_timing_report; PLX_ERR_SHAPE if buf_bytes is too small for all lines. */
PLX_API plx_status plx_timing_trace(plx_ctx* ctx, char* buf, size_t buf_bytes);

/* ---- adjacency set-up (Sec. 2.1 preprocessing + Sec. 5.1 double permutation) -----------------
 * plx_build_csr: src/dst are device int64[n_edges] node ids in [0, n), any order, either or
 * both directions, duplicates and self-loops allowed.  The graph is symmetrised, duplicates
 * and input loops dropped, exactly one self-loop per node added; d_u = number of stored
 * entries in row u (>= 1); value(u,v) = (float)(1.0 / sqrt((double)d_u * (double)d_v)).
 * perm_r / perm_c are device int64[n] with perm[old] = new (NULL = identity).  The handle
 * stores  A_fwd = P_r A^ P_c^T  and  A_bwd = A_fwd^T = P_c A^ P_r^T, both as CSR with strictly
 * ascending columns inside a row, plus the degrees in original id order.
 * Errors: PLX_ERR_INVALID for an id outside [0,n) or a permutation that is not a bijection
 * (detected on the GPU; the call waits for that answer); n >= 2^31, or 2 n_edges + n >= 2^31 (the
 * candidate entries before duplicates are dropped: both directions of every listed edge plus the
 * self-loops; an upper bound on the stored entries), is PLX_ERR_UNSUPPORTED. */
PLX_API plx_status plx_build_csr(plx_ctx* ctx, int64_t n, int64_t n_edges, const int64_t* src, const int64_t* dst,
                                 const int64_t* perm_r, const int64_t* perm_c, plx_csr** out);

/* plx_csr_import: adopt (copy) an already-built m x k block: device rowptr int64[m+1]
 * (rowptr[0] = 0, non-decreasing, rowptr[m] = nnz), col int32[nnz] in [0,k) ascending inside
 * a row, val fp32[nnz].  The transposed orientation is built by the library.  The structure
 * is checked on the GPU (PLX_ERR_INVALID if it is not as described). */
PLX_API plx_status plx_csr_import(plx_ctx* ctx, int64_t m, int64_t k, int64_t nnz, const int64_t* rowptr,
                                  const int32_t* col, const float* val, plx_csr** out);

/* m, k, nnz of the forward orientation (host outputs, any may be NULL). */
PLX_API plx_status plx_csr_dims(const plx_csr* csr, int64_t* m, int64_t* k, int64_t* nnz);

/* Copy one orientation out to caller-owned device arrays: transposed == 0 gives A_fwd
 * (rowptr int64[m+1], col int32[nnz], val fp32[nnz]); transposed != 0 gives A_bwd (rowptr
 * int64[k+1]).  deg (device int64[n], original id order) is written only for handles made by
 * plx_build_csr; pass NULL otherwise.  Any output pointer may be NULL to skip it. */
PLX_API plx_status plx_csr_export(plx_ctx* ctx, const plx_csr* csr, int transposed, int64_t* rowptr,
                                  int32_t* col, float* val, int64_t* deg);

/* Row-length summary of one orientation (host outputs, each int64[3] or NULL): the number of
 * rows, and of stored entries in those rows, with [0] fewer than 256, [1] 256..4095, [2] 4096 or
 * more entries.  Rows of bin [0] are handled by a group of lanes each; with column windows on
 * (the default) bins [1] and [2] go through the segment kernels, with the windows off bin [1]
 * takes one wavefront per row and only bin [2] is split.  For inspection, tests and the byte
 * accounting of a benchmark. */
PLX_API plx_status plx_csr_bins(const plx_csr* csr, int transposed, int64_t* rows, int64_t* entries);

PLX_API void plx_csr_destroy(plx_ctx* ctx, plx_csr* csr);

/* ---- sparse x dense (Eq. 2.1 and Eq. 2.7) -----------------------------------------------------
 * plx_spmm:   Y[m x d] = A_fwd X[k x d].      plx_spmm_t:   Y[k x d] = A_fwd^T X[m x d].
 * X, Y device, row-major, ldx, ldy >= d, Y fully overwritten (rows without entries become 0),
 * X and Y must not overlap.  128-bit gathers are used when X, Y are 16-byte aligned and ldx,
 * ldy are multiples of 16 bytes; other layouts take a narrower path with the same result.
 * No floating-point atomics: results are bit-identical from run to run. */
PLX_API plx_status plx_spmm(plx_ctx* ctx, const plx_csr* csr, const void* X, int64_t ldx, void* Y, int64_t ldy,
                            int64_t d, plx_dtype dtype);
PLX_API plx_status plx_spmm_t(plx_ctx* ctx, const plx_csr* csr, const void* X, int64_t ldx, void* Y, int64_t ldy,
                              int64_t d, plx_dtype dtype);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid it): plx_spmm (transposed == 0) or plx_spmm_t (transposed != 0) with the same
 * arguments and bit-identical results, except that the partial sums of split rows go to a fixed
 * 32 MiB buffer inside the library (one per GPU, held until the process ends) instead of the buffer
 * the handle holds for them (512 bytes per segment, allocated when the handle is built).  The call allocates nothing, frees nothing, records no timing events
 * (plx_timing_report does not list it) and does not wait.  Limit: (number of segments of the
 * orientation) x (floats per segment: d rounded up to a power-of-two number of 16-byte vectors, at
 * most 128 per pass) x 4 bytes <= 32 MiB, else PLX_ERR_UNSUPPORTED before anything is queued; a
 * handle without rows of 256 or more entries has no segments and always fits.  The buffer needs no
 * clearing (every segment's partial sums are fully rewritten before they are read), but all calls on
 * one GPU share it: two calls that overlap in time on the same GPU, from any context or stream, race.
 * PLX_ERR_DEVICE if the buffer's address could not be obtained when the context was created. */
PLX_API plx_status plx_spmm_static(plx_ctx* ctx, const plx_csr* csr, int transposed, const void* X, int64_t ldx,
                                   void* Y, int64_t ldy, int64_t d, plx_dtype dtype);

/* Blocked aggregation (Sec. 5.2: the adjacency is cut into row blocks, the product of each block
 * is formed -- and, on several GPUs, all-reduced -- separately, and the blocks are concatenated).
 * plx_csr_set_row_blocks re-bins both orientations into n_blocks (1..64) blocks of
 * ceil(rows / n_blocks) consecutive rows each (a set-up call: it waits, and moves the stored
 * entries).  plx_spmm_block then computes only the rows of one block of Y = A X (transposed == 0)
 * or Y = A^T X (transposed != 0); Y is the base of the WHOLE output matrix and rows outside the
 * block are not touched, so calling it for every block in any order gives exactly the result of
 * plx_spmm / plx_spmm_t (which keep working and walk over all blocks).
 * plx_csr_row_blocks reports the current blocking (host outputs).
 * Errors: PLX_ERR_INVALID for n_blocks outside 1..64 or a block index outside the current
 * blocking (nothing is changed); if plx_csr_set_row_blocks itself fails with PLX_ERR_OOM or
 * PLX_ERR_DEVICE the handle may be left half re-binned and must be destroyed. */
PLX_API plx_status plx_csr_set_row_blocks(plx_ctx* ctx, plx_csr* csr, int n_blocks);
PLX_API plx_status plx_csr_row_blocks(const plx_csr* csr, int transposed, int* n_blocks, int64_t* rows_per_block);
PLX_API plx_status plx_spmm_block(plx_ctx* ctx, const plx_csr* csr, int transposed, int block, const void* X,
                                  int64_t ldx, void* Y, int64_t ldy, int64_t d, plx_dtype dtype);

/* ---- dense x dense on the matrix cores (Eq. 2.2, 2.6, 2.5) --------------------------------------
 * plx_gemm_nn:  C[M x N] = A[M x K]   B[K x N]
 * plx_gemm_nt:  C[M x N] = A[M x K]   B[N x K]^T
 * plx_gemm_tn:  C[M x N] = A[R x M]^T B[R x N]     (reduction over the R rows, split over
 *               workgroups; partial sums are combined in a fixed order).  C is always fp32 for
 *               plx_gemm_tn; ws is device workspace of at least plx_gemm_tn_workspace bytes.
 * A, C of nn/nt have dtype `dtype`; the small operand B (a weight matrix) is always fp32.
 * All device, row-major.  PLX_BF16: products with K or N (tn: M or N) above 128, and every nt
 * product, need 16-byte aligned rows of their bf16 inputs (A; for tn A and B: base pointer
 * 16-byte aligned, leading dimension a multiple of 8) and leading dimensions below 2^22
 * elements, else PLX_ERR_UNSUPPORTED; the inputs are widened to fp32 (exact) and multiplied by the
 * fp32 matrix instructions.  The narrower nn and tn products take bf16 matrix instructions (B
 * rounded to bf16) with leading dimensions below 2^23.  The same holds for the products inside
 * the bf16 layer calls. */
PLX_API plx_status plx_gemm_nn(plx_ctx* ctx, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                               const float* B, int64_t ldb, void* C, int64_t ldc, plx_dtype dtype);
PLX_API plx_status plx_gemm_nt(plx_ctx* ctx, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                               const float* B, int64_t ldb, void* C, int64_t ldc, plx_dtype dtype);
PLX_API size_t plx_gemm_tn_workspace(int64_t R, int64_t M, int64_t N);
PLX_API plx_status plx_gemm_tn(plx_ctx* ctx, int64_t R, int64_t M, int64_t N, const void* A, int64_t lda,
                               const void* B, int64_t ldb, float* C, int64_t ldc, plx_dtype dtype,
                               void* ws, size_t ws_bytes);

/* ---- element-wise steps --------------------------------------------------------------------------
 * plx_relu (Eq. 2.3): F = max(Z, 0).  plx_relu_bwd (Eq. 2.4): dZ = dF where Z > 0, else 0.
 * rows x cols matrices, device; in-place (F == Z, dZ == dF) is allowed. */
PLX_API plx_status plx_relu(plx_ctx* ctx, int64_t rows, int64_t cols, const void* Z, int64_t ldz,
                            void* F, int64_t ldf, plx_dtype dtype);
PLX_API plx_status plx_relu_bwd(plx_ctx* ctx, int64_t rows, int64_t cols, const void* Z, int64_t ldz,
                                const void* dF, int64_t lddf, void* dZ, int64_t lddz, plx_dtype dtype);

/* Node-classification loss head (Sec. 2.1): mean softmax cross-entropy over all n rows of the
 * logits Z[n x c] against labels y (device int64[n], each in [0,c)); writes
 * dZ = (softmax(Z) - onehot(y)) / n and, if loss != NULL, the mean loss as one device fp32.
 * row_loss is device fp32[n] scratch (the per-row terms, summed in a fixed order). */
PLX_API plx_status plx_softmax_ce(plx_ctx* ctx, int64_t n, int64_t c, const void* Z, int64_t ldz, const int64_t* y,
                                  void* dZ, int64_t lddz, float* row_loss, float* loss, plx_dtype dtype);

/* ---- one GCN layer ---------------------------------------------------------------------------------
 * The adjacency used is A = A_fwd (transposed_A == 0, even layers) or A = A_bwd (transposed_A
 * != 0, odd layers), of shape ma x ka.  H is ka x din, W is din x dout (fp32), Z and F are
 * ma x dout.
 *
 * plx_gcn_layer_fwd:  Z = A H W (pre-activation) if Z != NULL; F = act(Z) if F != NULL; at least one
 *   of them must be given.  Storing only F saves one pass over the output: for ReLU the backward
 *   call accepts F in place of Z (F > 0 exactly where Z > 0).
 *   order AGG_FIRST : saved[ma x din] = A H (Eq. 2.1) then Z = saved W (Eq. 2.2); `saved` must
 *                     be given and is needed again by the backward call.
 *   order COMBINE_FIRST: T[ka x dout] = H W in the workspace, then Z = A T; `saved` is unused.
 *   order AUTO      : AGG_FIRST if din <= dout, else COMBINE_FIRST (so `saved` must be given
 *                     whenever din <= dout).  At equal widths both orders move the same bytes
 *                     through the sparse product, and aggregate-first applies Eq. 2.4 inside the
 *                     fused backward kernel instead of in a pass of its own.
 *   act RELU_BITS   : as RELU, but all the backward call needs of Z is kept, one bit per element: Z
 *                     (4-byte aligned, both Z and F required) receives uint32 words, ldz counts
 *                     words per row (>= ceil(dout / 32)); bit j % 32 of word j / 32 of row i is
 *                     [F[i][j] > 0], bits of columns >= dout inside the last word are 0.  The
 *                     backward call with act RELU_BITS reads the same words through `Z`, 1/32 of
 *                     the bytes of the value matrix.
 * plx_gcn_layer_bwd:  given dF (gradient wrt F, or wrt Z when act == NONE) computes
 *   dZ = dF * [Z > 0] (Eq. 2.4; `Z` may be the pre-activation or the ReLU output, only its sign is
 *   used; ignored when act == NONE), dW[din x dout] (fp32, Eq. 2.5) and, unless dH == NULL,
 *   dH[ka x din] (Eq. 2.6 + 2.7; the gradient wrt the layer input H).  H is read only in
 *   combine-first order, `saved` only in aggregate-first order.
 * ws: device workspace of at least plx_gcn_layer_workspace(...) bytes (same arguments), used
 * by both calls; its contents need not survive between them. */
PLX_API size_t plx_gcn_layer_workspace(const plx_csr* csr, int transposed_A, int64_t din, int64_t dout,
                                       plx_dtype dtype, plx_act act, plx_order order);
PLX_API plx_status plx_gcn_layer_fwd(plx_ctx* ctx, const plx_csr* csr, int transposed_A,
                                     const void* H, int64_t ldh, const float* W, int64_t ldw,
                                     int64_t din, int64_t dout, plx_dtype dtype, plx_act act, plx_order order,
                                     void* Z, int64_t ldz, void* F, int64_t ldf, void* saved, int64_t ldsaved,
                                     void* ws, size_t ws_bytes);
PLX_API plx_status plx_gcn_layer_bwd(plx_ctx* ctx, const plx_csr* csr, int transposed_A,
                                     const void* H, int64_t ldh, const float* W, int64_t ldw,
                                     const void* Z, int64_t ldz, const void* dF, int64_t lddf,
                                     const void* saved, int64_t ldsaved,
                                     int64_t din, int64_t dout, plx_dtype dtype, plx_act act, plx_order order,
                                     void* dH, int64_t lddh, float* dW, int64_t lddw, void* ws, size_t ws_bytes);

/* ---- forward of two consecutive layers without re-reading the activation between them --------------
 * Layer l+1 in combine-first order starts with T = F W (Eq. 2.2 first), a product over the rows of
 * layer l's output F.  plx_gcn_layer_fwd_chained is plx_gcn_layer_fwd of layer l that also writes
 * Tn[ma x dn] = F Wn (F: this layer's activated output, or Z when act == NONE; Wn[dout x dn] fp32,
 * the following layer's weights; Tn has dtype `dtype`), and plx_gcn_layer_fwd_from_t is the rest of
 * layer l+1: Z = A T, F = act(Z) for a given T[ka x dout].  F of layer l is still written (the
 * backward pass needs it) but not read again in the forward pass.
 * The extra product runs inside the kernel that writes F for fp32, aggregate-first order,
 * 32 < din <= 128, 32 < dout <= 128, din % 4 == 0, dn <= 16, 16-byte aligned rows of `saved`,
 * split products on; in every other case it is a product of its own after the layer (same result
 * up to rounding order, no saving).  With act != NONE F must be given.
 * Errors as plx_gcn_layer_fwd; PLX_ERR_INVALID if Tn / Wn / T is NULL or dn <= 0, PLX_ERR_SHAPE if
 * ldwn < dn, ldtn < dn or ldt < dout.  plx_gcn_layer_fwd_from_t uses no workspace. */
PLX_API plx_status plx_gcn_layer_fwd_chained(plx_ctx* ctx, const plx_csr* csr, int transposed_A,
                                             const void* H, int64_t ldh, const float* W, int64_t ldw,
                                             int64_t din, int64_t dout, plx_dtype dtype, plx_act act, plx_order order,
                                             void* Z, int64_t ldz, void* F, int64_t ldf, void* saved, int64_t ldsaved,
                                             const float* Wn, int64_t ldwn, int64_t dn, void* Tn, int64_t ldtn,
                                             void* ws, size_t ws_bytes);
PLX_API plx_status plx_gcn_layer_fwd_from_t(plx_ctx* ctx, const plx_csr* csr, int transposed_A,
                                            const void* T, int64_t ldt, int64_t dout, plx_dtype dtype, plx_act act,
                                            void* Z, int64_t ldz, void* F, int64_t ldf);

/* ---- backward of two consecutive layers without the gradient between them -------------------------
 * Layer l+1 in combine-first order computes T = H W, Z = A T (Eq. 2.1-2.2 in that order); its
 * backward pass is dT = A^T dZ, dW = H^T dT (Eq. 2.5) and dH = dT W^T (Eq. 2.6).  dH[ka x din] is
 * the dF of layer l and, on a graph of low degree, the largest matrix a step moves.  The two calls
 * below leave it out: the first stops before Eq. 2.6 and hands out dT (ka x dout, far narrower),
 * the second takes the pair (dT, W) of the following layer in place of dF and forms dF = dT W^T tile
 * by tile inside its fused backward kernel.
 *
 * plx_gcn_layer_bwd_dt: as plx_gcn_layer_bwd in combine-first order with dH == NULL, except that
 *   dT[ka x dout] (dtype `dtype`, device, caller's) receives A^T (dF * [Z > 0]).  W is not read.
 *   ws: plx_gcn_layer_workspace(..., PLX_ORDER_COMBINE_FIRST) bytes.
 * plx_gcn_layer_bwd_chained: as plx_gcn_layer_bwd with dF = dTn Wn^T, where dTn[ma x dn] (dtype
 *   `dtype`) is the dT of the following layer and Wn[dout x dn] (fp32) its weight matrix.  The
 *   product is formed inside the fused kernel for fp32, aggregate-first order, 32 < din <= 128,
 *   64 < dout <= 128, dn <= 32, no mask or the sign-bit mask, 16-byte aligned rows of `saved` and
 *   dTn, split products on; in every other case it is formed once in the workspace and the call
 *   proceeds as plx_gcn_layer_bwd would (same results, no saving).
 *   ws: plx_gcn_layer_bwd_chained_workspace(...) bytes: the layer workspace, plus room for that
 *   formed gradient unless the shapes (and the context's split-product switch) put the product
 *   inside the kernel.  The query takes 16-byte aligned rows for granted; if the call then meets
 *   unaligned ones and the workspace lacks the room, it fails with PLX_ERR_SHAPE and names the size.
 * Errors as plx_gcn_layer_bwd; PLX_ERR_INVALID if dT / dTn / Wn is NULL or dn <= 0, PLX_ERR_SHAPE
 * if lddt < dout, lddtn < dn or ldwn < dn. */
PLX_API plx_status plx_gcn_layer_bwd_dt(plx_ctx* ctx, const plx_csr* csr, int transposed_A,
                                        const void* H, int64_t ldh, const void* Z, int64_t ldz,
                                        const void* dF, int64_t lddf, int64_t din, int64_t dout,
                                        plx_dtype dtype, plx_act act, void* dT, int64_t lddt,
                                        float* dW, int64_t lddw, void* ws, size_t ws_bytes);
PLX_API size_t plx_gcn_layer_bwd_chained_workspace(const plx_ctx* ctx, const plx_csr* csr, int transposed_A,
                                                   int64_t din, int64_t dout, int64_t dn,
                                                   plx_dtype dtype, plx_act act, plx_order order);
PLX_API plx_status plx_gcn_layer_bwd_chained(plx_ctx* ctx, const plx_csr* csr, int transposed_A,
                                             const void* H, int64_t ldh, const float* W, int64_t ldw,
                                             const void* Z, int64_t ldz, const void* dTn, int64_t lddtn,
                                             const float* Wn, int64_t ldwn, int64_t dn,
                                             const void* saved, int64_t ldsaved,
                                             int64_t din, int64_t dout, plx_dtype dtype, plx_act act, plx_order order,
                                             void* dH, int64_t lddh, float* dW, int64_t lddw, void* ws, size_t ws_bytes);

/* What a sequencer of several layers should ask of the calls above for one layer, so that it holds no copy of the
 * kernels' shape limits.  The layer is din -> dout in `order`; dn > 0 is the output width of a following layer that
 * runs in `next_order` (dn == 0: no following layer, or it is not to be paired); keep_values != 0 says the caller
 * keeps the ReLU mask as a value matrix (PLX_ACT_RELU) whatever is possible.  Host outputs (any may be NULL):
 *   agg_first: the order PLX_ORDER_AUTO / `order` resolves to is aggregate-first;
 *   sign_bits: PLX_ACT_RELU_BITS is worth using (the layer's own dense kernels write the bits on the fly);
 *   chain_fwd: plx_gcn_layer_fwd_chained + plx_gcn_layer_fwd_from_t form T = F Wn inside this layer's product;
 *   chain_bwd: plx_gcn_layer_bwd_dt + plx_gcn_layer_bwd_chained form the gradient inside this layer's fused kernel.
 * The answers depend on the context's split-product switch and assume 16-byte aligned rows.  PLX_ERR_INVALID for a
 * NULL context, non-positive widths or unknown enums. */
PLX_API plx_status plx_gcn_layer_plan(const plx_ctx* ctx, int64_t din, int64_t dout, int64_t dn, plx_dtype dtype,
                                      plx_order order, plx_order next_order, int keep_values, int* agg_first,
                                      int* sign_bits, int* chain_fwd, int* chain_bwd);

#ifdef __cplusplus
}
#endif
#endif /* PLX_H */
