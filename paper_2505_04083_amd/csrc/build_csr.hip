// One-time adjacency set-up on the GPU (paper Sec. 2.1 preprocessing; Sec. 5.1, Eq. 5.3-5.4):
// symmetrise, drop duplicates and input loops, add one self-loop per node, relabel rows by
// P_r and columns by P_c, sort into canonical CSR, value = 1/sqrt(d_u d_v); then the
// transposed orientation and the row binning the sparse kernels use.
//
// All structure work is integer work: 64-bit keys row*n+col, device radix sort (rocPRIM),
// neighbour comparison for duplicates, prefix sums for compaction and row pointers.
#include "plx_internal.h"

#include <algorithm>
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_scan.hpp>

namespace plx {
namespace {

constexpr int kThreads = 256;
inline unsigned grid_for(int64_t n, int per_block = kThreads) {
    int64_t g = ceil_div(n, per_block);
    return (unsigned)std::max<int64_t>(1, std::min<int64_t>(g, 1 << 20));
}

#define GRID_STRIDE(i, n) \
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < (n); i += (int64_t)gridDim.x * blockDim.x)

enum : int { kFlagBadId = 1, kFlagBadPerm = 2, kFlagBadStruct = 4 };

__global__ void k_check_ids(int64_t n, int64_t ne, const int64_t* src, const int64_t* dst, int* flags) {
    GRID_STRIDE(e, ne) {
        int64_t u = src[e], v = dst[e];
        if (u < 0 || v < 0 || u >= n || v >= n) atomicOr(flags, kFlagBadId);
    }
}

__global__ void k_mark_perm(int64_t n, const int64_t* perm, int* hits, int* flags) {
    GRID_STRIDE(i, n) {
        int64_t p = perm[i];
        if (p < 0 || p >= n) atomicOr(flags, kFlagBadPerm);
        else atomicAdd(&hits[p], 1);
    }
}

__global__ void k_check_hits(int64_t n, const int* hits, int* flags) {
    GRID_STRIDE(i, n) if (hits[i] != 1) atomicOr(flags, kFlagBadPerm);
}

// keys of both directions of every non-loop edge plus one self-loop per node, in permuted ids
__global__ void k_make_keys(int64_t n, int64_t ne, const int64_t* src, const int64_t* dst, const int64_t* pr,
                            const int64_t* pc, uint64_t* keys, uint64_t sentinel) {
    GRID_STRIDE(i, ne + n) {
        if (i < ne) {
            int64_t u = src[i], v = dst[i];
            if (u == v) {
                keys[2 * i] = sentinel; keys[2 * i + 1] = sentinel;
            } else {
                uint64_t ur = pr ? pr[u] : u, uc = pc ? pc[u] : u;
                uint64_t vr = pr ? pr[v] : v, vc = pc ? pc[v] : v;
                keys[2 * i] = ur * (uint64_t)n + vc;
                keys[2 * i + 1] = vr * (uint64_t)n + uc;
            }
        } else {
            int64_t u = i - ne;
            uint64_t ur = pr ? pr[u] : u, uc = pc ? pc[u] : u;
            keys[2 * ne + u] = ur * (uint64_t)n + uc;
        }
    }
}

__global__ void k_flag_unique(int64_t count, const uint64_t* keys, uint64_t sentinel, uint32_t* flag) {
    GRID_STRIDE(i, count) {
        uint64_t k = keys[i];
        flag[i] = (k != sentinel && (i == 0 || keys[i - 1] != k)) ? 1u : 0u;
    }
}

// compact the unique keys into (row, col) and count the row lengths
__global__ void k_scatter_unique(int64_t count, const uint64_t* keys, const uint32_t* flag, const uint32_t* pos,
                                 uint64_t n, int32_t* row, int32_t* col, unsigned int* rowcount) {
    GRID_STRIDE(i, count) {
        if (!flag[i]) continue;
        uint64_t k = keys[i];
        uint32_t p = pos[i];
        int32_t r = (int32_t)(k / n), c = (int32_t)(k % n);
        row[p] = r; col[p] = c;
        atomicAdd(&rowcount[r], 1u);
    }
}

__global__ void k_widen_counts(int64_t n, const unsigned int* cnt, int64_t* out) {
    GRID_STRIDE(i, n) out[i] = (int64_t)cnt[i];
}

// deg (original ids) and the column-side degree table from the permuted-row lengths
__global__ void k_degrees(int64_t n, const int64_t* rowptr, const int64_t* pr, const int64_t* pc, int64_t* deg,
                          int64_t* deg_c) {
    GRID_STRIDE(u, n) {
        int64_t r = pr ? pr[u] : u;
        int64_t d = rowptr[r + 1] - rowptr[r];
        deg[u] = d;
        deg_c[pc ? pc[u] : u] = d;
    }
}

// value = (float)(1 / sqrt(d_row * d_col)), every step a correctly rounded fp64 operation
__global__ void k_values(int64_t nnz, const int32_t* row, const int32_t* col, const int64_t* rowptr,
                         const int64_t* deg_c, float* val) {
    GRID_STRIDE(e, nnz) {
        int32_t r = row[e];
        double dr = (double)(rowptr[r + 1] - rowptr[r]);
        double dc = (double)deg_c[col[e]];
        val[e] = (float)(1.0 / sqrt(dr * dc));
    }
}

// ---- transposition of a CSR orientation --------------------------------------------------------

__global__ void k_expand_rows(int64_t rows, int64_t nnz, const int64_t* rowptr, int32_t* row) {
    GRID_STRIDE(e, nnz) {
        int64_t lo = 0, hi = rows;            // last row r with rowptr[r] <= e
        while (hi - lo > 1) {
            int64_t mid = (lo + hi) >> 1;
            if (rowptr[mid] <= e) lo = mid; else hi = mid;
        }
        row[e] = (int32_t)lo;
    }
}

__global__ void k_transpose_keys(int64_t nnz, const int32_t* row, const int32_t* col, uint64_t rows,
                                 uint64_t* keys, unsigned int* colcount) {
    GRID_STRIDE(e, nnz) {
        keys[e] = (uint64_t)col[e] * rows + (uint64_t)row[e];
        atomicAdd(&colcount[col[e]], 1u);
    }
}

__global__ void k_keys_to_cols(int64_t nnz, const uint64_t* keys, uint64_t rows, int32_t* col) {
    GRID_STRIDE(e, nnz) col[e] = (int32_t)(keys[e] % rows);
}

// ---- structure check of an imported block ---------------------------------------------------------

__global__ void k_check_rowptr(int64_t m, int64_t nnz, const int64_t* rowptr, int* flags) {
    GRID_STRIDE(i, m + 1) {
        int64_t a = rowptr[i];
        if (a < 0 || a > nnz) atomicOr(flags, kFlagBadStruct);
        if (i == 0 && a != 0) atomicOr(flags, kFlagBadStruct);
        if (i == m && a != nnz) atomicOr(flags, kFlagBadStruct);
        if (i < m && rowptr[i + 1] < a) atomicOr(flags, kFlagBadStruct);
    }
}

__global__ void k_check_cols(int64_t nnz, int64_t k, const int32_t* row, const int32_t* col, int* flags) {
    GRID_STRIDE(e, nnz) {
        int32_t c = col[e];
        if (c < 0 || c >= k) atomicOr(flags, kFlagBadStruct);
        if (e > 0 && row[e - 1] == row[e] && col[e - 1] >= c) atomicOr(flags, kFlagBadStruct);
    }
}

// ---- binning ------------------------------------------------------------------------------------------

__device__ __forceinline__ int length_class(int64_t len) {
    return len <= 0 ? 0 : 64 - __clzll((unsigned long long)len);   // 1 + floor(log2 len)
}

// sort key of a row = block * 64 + length class; histograms of rows and entries per key
__global__ void k_row_class(int64_t rows, const int64_t* rowptr, int64_t rows_per_block, int n_keys, uint16_t* key,
                            int32_t* ids, unsigned int* hist, unsigned long long* hist_nnz) {
    extern __shared__ unsigned long long sh[];          // [n_keys] entry counts, then [n_keys] row counts
    unsigned long long* hn = sh;
    unsigned int* h = reinterpret_cast<unsigned int*>(sh + n_keys);
    for (int c = threadIdx.x; c < n_keys; c += blockDim.x) { h[c] = 0; hn[c] = 0; }
    __syncthreads();
    GRID_STRIDE(r, rows) {
        int64_t len = rowptr[r + 1] - rowptr[r];
        int k = (int)(r / rows_per_block) * 64 + length_class(len);
        key[r] = (uint16_t)k;
        ids[r] = (int32_t)r;
        atomicAdd(&h[k], 1u);
        atomicAdd(&hn[k], (unsigned long long)len);
    }
    __syncthreads();
    for (int c = threadIdx.x; c < n_keys; c += blockDim.x)
        if (h[c]) { atomicAdd(&hist[c], h[c]); atomicAdd(&hist_nnz[c], hn[c]); }
}

// ---- segments of the long rows ----------------------------------------------------------------------
// first entry of [lo, hi) whose column is >= c (columns ascend inside a row)
__device__ __forceinline__ int32_t lower_bound_col(const int32_t* __restrict__ col, int32_t lo, int32_t hi, int64_t c) {
    while (lo < hi) {
        const int32_t mid = lo + ((hi - lo) >> 1);
        if (col[mid] < c) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// entry range of long row q inside column window w
__device__ __forceinline__ void window_range(const int32_t* __restrict__ bptr, const int32_t* __restrict__ col, int32_t slot,
                                             int w, int n_windows, int64_t win_cols, int32_t* lo, int32_t* hi) {
    const int32_t b0 = bptr[slot], b1 = bptr[slot + 1];
    *lo = w == 0 ? b0 : lower_bound_col(col, b0, b1, (int64_t)w * win_cols);
    *hi = w + 1 == n_windows ? b1 : lower_bound_col(col, b0, b1, (int64_t)(w + 1) * win_cols);
}

// cnt[q * n_windows + w] = number of segments of (long row q, window w)
__global__ void k_seg_count(int64_t n_long, const int32_t* __restrict__ long_slot, const int32_t* __restrict__ bptr,
                            const int32_t* __restrict__ col, int n_windows, int64_t win_cols, int32_t seg_max,
                            int32_t* __restrict__ cnt) {
    GRID_STRIDE(i, n_long * n_windows) {
        const int64_t q = i / n_windows;
        const int w = (int)(i % n_windows);
        int32_t lo, hi;
        window_range(bptr, col, long_slot[q], w, n_windows, win_cols, &lo, &hi);
        cnt[i] = (hi - lo + seg_max - 1) / seg_max;
    }
}

// segment arrays; first[i] = exclusive scan of cnt (row-major: the order partial sums are added in)
__global__ void k_seg_fill(int64_t n_long, const int32_t* __restrict__ long_slot, const int32_t* __restrict__ row_order,
                           const int32_t* __restrict__ bptr, const int32_t* __restrict__ col, int n_windows, int64_t win_cols,
                           int32_t seg_max, const int32_t* __restrict__ first, int64_t rows_per_block,
                           int32_t* __restrict__ long_row, int32_t* __restrict__ long_seg0, int64_t* __restrict__ seg_lo,
                           int32_t* __restrict__ seg_len, uint16_t* __restrict__ key, int32_t* __restrict__ id) {
    GRID_STRIDE(i, n_long * n_windows) {
        const int64_t q = i / n_windows;
        const int w = (int)(i % n_windows);
        const int32_t slot = long_slot[q], row = row_order[slot];
        if (w == 0) { long_row[q] = row; long_seg0[q] = first[i]; }
        int32_t lo, hi;
        window_range(bptr, col, slot, w, n_windows, win_cols, &lo, &hi);
        const uint16_t k = (uint16_t)((row / rows_per_block) * n_windows + w);
        int32_t s2 = first[i];
        for (int32_t e = lo; e < hi; e += seg_max, ++s2) {
            seg_lo[s2] = e;
            seg_len[s2] = hi - e < seg_max ? hi - e : seg_max;
            key[s2] = k;
            id[s2] = s2;
        }
    }
}

// the segments in launch order, one 16-byte record each
__global__ void k_seg_desc(int64_t n_seg, const int32_t* __restrict__ launch, const int64_t* __restrict__ seg_lo,
                           const int32_t* __restrict__ seg_len, int4* __restrict__ desc) {
    GRID_STRIDE(pos, n_seg) {
        const int32_t seg = launch[pos];
        desc[pos] = make_int4((int32_t)seg_lo[seg], seg_len[seg], seg, 0);
    }
}

// length of the row held by each slot of the binned order (slot `rows` gets 0 for the scan)
__global__ void k_slot_len(int64_t rows, const int32_t* row_order, const int64_t* rowptr, int32_t* len) {
    GRID_STRIDE(s, rows + 1) {
        if (s < rows) { int32_t r = row_order[s]; len[s] = (int32_t)(rowptr[r + 1] - rowptr[r]); }
        else len[s] = 0;
    }
}

// Entry e of the binned storage belongs to slot s (bptr[s] <= e < bptr[s+1]); its place in the
// canonical CSR is rowptr[row_order[s]] + (e - bptr[s]).  to_binned copies canonical -> binned,
// otherwise binned -> canonical.
__global__ void k_move_entries(int64_t rows, int64_t nnz, const int32_t* bptr, const int32_t* row_order,
                               const int64_t* rowptr, const int32_t* col_in, const float* val_in, int32_t* col_out,
                               float* val_out, int to_binned) {
    GRID_STRIDE(e, nnz) {
        int64_t lo = 0, hi = rows;            // last slot with bptr[slot] <= e
        while (hi - lo > 1) {
            int64_t mid = (lo + hi) >> 1;
            if (bptr[mid] <= e) lo = mid; else hi = mid;
        }
        const int64_t canon = rowptr[row_order[lo]] + (e - bptr[lo]);
        const int64_t src = to_binned ? canon : e, dst = to_binned ? e : canon;
        if (col_in) col_out[dst] = col_in[src];
        if (val_in) val_out[dst] = val_in[src];
    }
}

template <typename T>
plx_status scan_exclusive(plx_ctx* ctx, TempPool& pool, const T* in, T* out, size_t count) {
    size_t bytes = 0;
    PLX_HIP(ctx, rocprim::exclusive_scan(nullptr, bytes, in, out, T(0), count, rocprim::plus<T>(), ctx->stream));
    void* tmp = pool.get<char>(bytes);
    if (!tmp) return PLX_ERR_OOM;
    PLX_HIP(ctx, rocprim::exclusive_scan(tmp, bytes, in, out, T(0), count, rocprim::plus<T>(), ctx->stream));
    return PLX_OK;
}

int bit_length(uint64_t x) { int b = 0; while (x) { ++b; x >>= 1; } return b; }

// rowptr[0..rows] from per-row counts (counts array has rows + 1 entries, last one ignored/zero)
plx_status counts_to_rowptr(plx_ctx* ctx, TempPool& pool, const unsigned int* counts, int64_t rows, int64_t* rowptr) {
    int64_t* wide = pool.get<int64_t>(rows + 1);
    if (!wide) return PLX_ERR_OOM;
    PLX_HIP(ctx, hipMemsetAsync(wide + rows, 0, sizeof(int64_t), ctx->stream));
    k_widen_counts<<<grid_for(rows), kThreads, 0, ctx->stream>>>(rows, counts, wide);
    return scan_exclusive<int64_t>(ctx, pool, wide, rowptr, (size_t)rows + 1);
}

// dst = transpose of src (src complete except binning); row ids of src's entries in `src_row`
plx_status transpose_orient(plx_ctx* ctx, const Orient& src, const int32_t* src_row, Orient& dst) {
    TempPool pool(ctx);
    dst.rows = src.cols; dst.cols = src.rows; dst.nnz = src.nnz;
    dst.rowptr = static_cast<int64_t*>(dev_alloc(ctx, sizeof(int64_t) * (dst.rows + 1)));
    dst.col = static_cast<int32_t*>(dev_alloc(ctx, sizeof(int32_t) * std::max<int64_t>(1, dst.nnz)));
    dst.val = static_cast<float*>(dev_alloc(ctx, sizeof(float) * std::max<int64_t>(1, dst.nnz)));
    if (!dst.rowptr || !dst.col || !dst.val) return PLX_ERR_OOM;
    unsigned int* colcount = pool.get<unsigned int>(dst.rows + 1);
    uint64_t* keys = pool.get<uint64_t>(src.nnz);
    uint64_t* keys_sorted = pool.get<uint64_t>(src.nnz);
    if (!colcount || !keys || !keys_sorted) return PLX_ERR_OOM;
    PLX_HIP(ctx, hipMemsetAsync(colcount, 0, sizeof(unsigned int) * (dst.rows + 1), ctx->stream));
    if (src.nnz > 0) {
        k_transpose_keys<<<grid_for(src.nnz), kThreads, 0, ctx->stream>>>(src.nnz, src_row, src.col, (uint64_t)src.rows,
                                                                           keys, colcount);
        int bits = std::max(1, bit_length((uint64_t)src.cols * (uint64_t)src.rows));
        size_t bytes = 0;
        PLX_HIP(ctx, rocprim::radix_sort_pairs(nullptr, bytes, keys, keys_sorted, src.val, dst.val, (size_t)src.nnz, 0,
                                               bits, ctx->stream));
        void* tmp = pool.get<char>(bytes);
        if (!tmp) return PLX_ERR_OOM;
        PLX_HIP(ctx, rocprim::radix_sort_pairs(tmp, bytes, keys, keys_sorted, src.val, dst.val, (size_t)src.nnz, 0,
                                               bits, ctx->stream));
        k_keys_to_cols<<<grid_for(src.nnz), kThreads, 0, ctx->stream>>>(src.nnz, keys_sorted, (uint64_t)src.rows, dst.col);
    }
    PLX_TRY(counts_to_rowptr(ctx, pool, colcount, dst.rows, dst.rowptr));
    PLX_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return PLX_OK;
}

}  // namespace

void segment_policy(const plx_ctx* ctx, int64_t rows, int64_t cols, int64_t nnz, int* n_windows, int* long_class, int32_t* seg_max) {
    (void)rows; (void)nnz;
    *seg_max = (int32_t)kSegLen;
    if (ctx->n_windows <= 1 || cols < 2 * ctx->n_windows) {     // no windows: only the very long rows are split
        *n_windows = 1;
        *long_class = kLongClass;
        return;
    }
    *n_windows = ctx->n_windows;
    *long_class = kSubwaveMaxClass + 1;         // every row that is not handled by a group of lanes
}

plx_status build_bins(plx_ctx* ctx, Orient& o, int n_blocks) {
    TempPool pool(ctx);
    if (n_blocks < 1) n_blocks = 1;
    o.n_blocks = n_blocks;
    o.rows_per_block = std::max<int64_t>(1, ceil_div(o.rows, n_blocks));
    const int n_keys = n_blocks * 64;
    o.row_order = static_cast<int32_t*>(dev_alloc(ctx, sizeof(int32_t) * std::max<int64_t>(1, o.rows)));
    if (!o.row_order) return PLX_ERR_OOM;
    uint16_t* key = pool.get<uint16_t>(o.rows);
    uint16_t* key_sorted = pool.get<uint16_t>(o.rows);
    int32_t* ids = pool.get<int32_t>(o.rows);
    unsigned int* hist = pool.get<unsigned int>(n_keys);
    unsigned long long* hist_nnz = pool.get<unsigned long long>(n_keys);
    if (!key || !key_sorted || !ids || !hist || !hist_nnz) return PLX_ERR_OOM;
    PLX_HIP(ctx, hipMemsetAsync(hist, 0, sizeof(unsigned int) * n_keys, ctx->stream));
    PLX_HIP(ctx, hipMemsetAsync(hist_nnz, 0, sizeof(unsigned long long) * n_keys, ctx->stream));
    std::vector<unsigned int> h(n_keys, 0);
    std::vector<unsigned long long> hn(n_keys, 0);
    if (o.rows > 0) {
        const size_t lds = (sizeof(unsigned long long) + sizeof(unsigned int)) * n_keys;
        k_row_class<<<std::min(grid_for(o.rows), 2048u), kThreads, lds, ctx->stream>>>(o.rows, o.rowptr, o.rows_per_block, n_keys,
                                                                                        key, ids, hist, hist_nnz);
        const int bits = std::max(6, bit_length((uint64_t)n_keys - 1));
        size_t bytes = 0;   // stable sort by (block, class): ids stay ascending inside a class
        PLX_HIP(ctx, rocprim::radix_sort_pairs(nullptr, bytes, key, key_sorted, ids, o.row_order, (size_t)o.rows, 0, bits,
                                               ctx->stream));
        void* tmp = pool.get<char>(bytes);
        if (!tmp) return PLX_ERR_OOM;
        PLX_HIP(ctx, rocprim::radix_sort_pairs(tmp, bytes, key, key_sorted, ids, o.row_order, (size_t)o.rows, 0, bits,
                                               ctx->stream));
    }
    PLX_HIP(ctx, hipMemcpyAsync(h.data(), hist, sizeof(unsigned int) * n_keys, hipMemcpyDeviceToHost, ctx->stream));
    PLX_HIP(ctx, hipMemcpyAsync(hn.data(), hist_nnz, sizeof(unsigned long long) * n_keys, hipMemcpyDeviceToHost, ctx->stream));
    PLX_HIP(ctx, hipStreamSynchronize(ctx->stream));
    o.boff.assign((size_t)n_blocks * (kNumClasses + 1), 0);
    o.bnnz.assign((size_t)n_blocks * kNumClasses, 0);
    int64_t run = 0;
    for (int b = 0; b < n_blocks; ++b) {
        for (int c = 0; c < kNumClasses; ++c) {
            o.boff[(size_t)b * (kNumClasses + 1) + c] = run;
            run += h[b * 64 + c];
            o.bnnz[(size_t)b * kNumClasses + c] = (int64_t)hn[b * 64 + c];
        }
        o.boff[(size_t)b * (kNumClasses + 1) + kNumClasses] = run;
    }

    // binned storage: slot pointers, then move the entries so that the rows of a bin are contiguous
    o.bptr = static_cast<int32_t*>(dev_alloc(ctx, sizeof(int32_t) * (o.rows + 1)));
    if (!o.bptr) return PLX_ERR_OOM;
    {
        int32_t* len = pool.get<int32_t>(o.rows + 1);
        if (!len) return PLX_ERR_OOM;
        k_slot_len<<<grid_for(o.rows + 1), kThreads, 0, ctx->stream>>>(o.rows, o.row_order, o.rowptr, len);
        PLX_TRY(scan_exclusive<int32_t>(ctx, pool, len, o.bptr, (size_t)o.rows + 1));
        if (o.nnz > 0) {
            int32_t* col_b = static_cast<int32_t*>(dev_alloc(ctx, sizeof(int32_t) * o.nnz));
            float* val_b = static_cast<float*>(dev_alloc(ctx, sizeof(float) * o.nnz));
            if (!col_b || !val_b) { dev_free(ctx, col_b); dev_free(ctx, val_b); return PLX_ERR_OOM; }
            k_move_entries<<<grid_for(o.nnz), kThreads, 0, ctx->stream>>>(o.rows, o.nnz, o.bptr, o.row_order, o.rowptr,
                                                                          o.col, o.val, col_b, val_b, 1);
            PLX_HIP(ctx, hipStreamSynchronize(ctx->stream));
            dev_free(ctx, o.col); dev_free(ctx, o.val);
            o.col = col_b; o.val = val_b;
        }
    }

    // long rows -> segments, in binned coordinates
    segment_policy(ctx, o.rows, o.cols, o.nnz, &o.n_windows, &o.long_class, &o.seg_max);
    const int NW = o.n_windows;
    const int64_t win_cols = std::max<int64_t>(1, ceil_div(o.cols, NW));
    o.long0.assign(n_blocks + 1, 0);
    o.seg0b.assign(n_blocks + 1, 0);
    std::vector<int32_t> long_slot_h;
    for (int b = 0; b < n_blocks; ++b) {
        o.long0[b] = (int64_t)long_slot_h.size();
        for (int64_t sl = o.off(b, o.long_class); sl < o.off(b, kNumClasses); ++sl) long_slot_h.push_back((int32_t)sl);
    }
    o.long0[n_blocks] = (int64_t)long_slot_h.size();
    o.n_long = (int64_t)long_slot_h.size();
    o.n_seg = 0;
    if (o.n_long > 0) {
        if (o.n_long * NW >= (int64_t(1) << 31)) return fail(ctx, PLX_ERR_UNSUPPORTED, "too many (long row, window) pairs");
        const int64_t pairs = o.n_long * NW;
        int32_t* long_slot = pool.get<int32_t>(o.n_long);
        int32_t* cnt = pool.get<int32_t>(pairs + 1);
        int32_t* first = pool.get<int32_t>(pairs + 1);
        if (!long_slot || !cnt || !first) return PLX_ERR_OOM;
        PLX_HIP(ctx, hipMemcpyAsync(long_slot, long_slot_h.data(), sizeof(int32_t) * o.n_long, hipMemcpyHostToDevice, ctx->stream));
        PLX_HIP(ctx, hipMemsetAsync(cnt + pairs, 0, sizeof(int32_t), ctx->stream));
        k_seg_count<<<grid_for(pairs), kThreads, 0, ctx->stream>>>(o.n_long, long_slot, o.bptr, o.col, NW, win_cols, o.seg_max, cnt);
        PLX_TRY(scan_exclusive<int32_t>(ctx, pool, cnt, first, (size_t)pairs + 1));
        int32_t n_seg32 = 0;
        PLX_HIP(ctx, hipMemcpyAsync(&n_seg32, first + pairs, sizeof(int32_t), hipMemcpyDeviceToHost, ctx->stream));
        PLX_HIP(ctx, hipStreamSynchronize(ctx->stream));      // also: long_slot_h has been read
        o.n_seg = n_seg32;
        const int64_t ns = std::max<int64_t>(1, o.n_seg);
        o.long_row = static_cast<int32_t*>(dev_alloc(ctx, sizeof(int32_t) * o.n_long));
        o.long_seg0 = static_cast<int32_t*>(dev_alloc(ctx, sizeof(int32_t) * (o.n_long + 1)));
        o.seg_lo = static_cast<int64_t*>(dev_alloc(ctx, sizeof(int64_t) * ns));
        o.seg_len = static_cast<int32_t*>(dev_alloc(ctx, sizeof(int32_t) * ns));
        o.seg_launch = static_cast<int32_t*>(dev_alloc(ctx, sizeof(int32_t) * ns));
        uint16_t* skey = pool.get<uint16_t>(ns);
        uint16_t* skey_sorted = pool.get<uint16_t>(ns);
        int32_t* sid = pool.get<int32_t>(ns);
        if (!o.long_row || !o.long_seg0 || !o.seg_lo || !o.seg_len || !o.seg_launch || !skey || !skey_sorted || !sid)
            return PLX_ERR_OOM;
        k_seg_fill<<<grid_for(pairs), kThreads, 0, ctx->stream>>>(o.n_long, long_slot, o.row_order, o.bptr, o.col, NW, win_cols,
                                                                   o.seg_max, first, o.rows_per_block, o.long_row, o.long_seg0,
                                                                   o.seg_lo, o.seg_len, skey, sid);
        PLX_HIP(ctx, hipMemcpyAsync(o.long_seg0 + o.n_long, first + pairs, sizeof(int32_t), hipMemcpyDeviceToDevice, ctx->stream));
        if (o.n_seg > 0) {                                    // launch order: stable sort of the segment ids by (block, window)
            const int bits = std::max(1, bit_length((uint64_t)n_blocks * NW - 1));
            size_t bytes = 0;
            PLX_HIP(ctx, rocprim::radix_sort_pairs(nullptr, bytes, skey, skey_sorted, sid, o.seg_launch, (size_t)o.n_seg, 0, bits,
                                                   ctx->stream));
            void* tmp = pool.get<char>(bytes);
            if (!tmp) return PLX_ERR_OOM;
            PLX_HIP(ctx, rocprim::radix_sort_pairs(tmp, bytes, skey, skey_sorted, sid, o.seg_launch, (size_t)o.n_seg, 0, bits,
                                                   ctx->stream));
        }
        for (int b = 0; b <= n_blocks; ++b) {                 // first segment of every block
            int32_t v = n_seg32;
            if (o.long0[b] < o.n_long)
                PLX_HIP(ctx, hipMemcpyAsync(&v, first + o.long0[b] * NW, sizeof(int32_t), hipMemcpyDeviceToHost, ctx->stream));
            PLX_HIP(ctx, hipStreamSynchronize(ctx->stream));
            o.seg0b[b] = v;
        }
    }
    if (o.n_seg > 0) {
        o.part = static_cast<float*>(dev_alloc(ctx, sizeof(float) * (size_t)o.n_seg * kPartFloats));
        o.seg_desc = static_cast<int4*>(dev_alloc(ctx, sizeof(int4) * (size_t)o.n_seg));
        if (!o.part || !o.seg_desc) return PLX_ERR_OOM;
        k_seg_desc<<<grid_for(o.n_seg), kThreads, 0, ctx->stream>>>(o.n_seg, o.seg_launch, o.seg_lo, o.seg_len, o.seg_desc);
    }
    PLX_HIP(ctx, hipStreamSynchronize(ctx->stream));
    PLX_HIP(ctx, hipGetLastError());
    return PLX_OK;
}

plx_status unbin(plx_ctx* ctx, Orient& o) {
    if (o.nnz > 0) {
        int32_t* col_c = static_cast<int32_t*>(dev_alloc(ctx, sizeof(int32_t) * o.nnz));
        float* val_c = static_cast<float*>(dev_alloc(ctx, sizeof(float) * o.nnz));
        if (!col_c || !val_c) { dev_free(ctx, col_c); dev_free(ctx, val_c); return PLX_ERR_OOM; }
        k_move_entries<<<grid_for(o.nnz), kThreads, 0, ctx->stream>>>(o.rows, o.nnz, o.bptr, o.row_order, o.rowptr, o.col,
                                                                      o.val, col_c, val_c, 0);
        PLX_HIP(ctx, hipStreamSynchronize(ctx->stream));
        dev_free(ctx, o.col); dev_free(ctx, o.val);
        o.col = col_c; o.val = val_c;
    } else {
        PLX_HIP(ctx, hipStreamSynchronize(ctx->stream));
    }
    dev_free(ctx, o.row_order); dev_free(ctx, o.bptr);
    dev_free(ctx, o.long_row); dev_free(ctx, o.long_seg0); dev_free(ctx, o.seg_lo); dev_free(ctx, o.seg_len);
    dev_free(ctx, o.seg_launch); o.seg_launch = nullptr;
    dev_free(ctx, o.part); o.part = nullptr;
    dev_free(ctx, o.seg_desc); o.seg_desc = nullptr;
    o.row_order = nullptr; o.bptr = nullptr; o.long_row = nullptr; o.long_seg0 = nullptr; o.seg_lo = nullptr; o.seg_len = nullptr;
    o.n_long = o.n_seg = 0;
    return PLX_OK;
}

plx_status export_entries(plx_ctx* ctx, const Orient& o, int32_t* col, float* val) {
    if (o.nnz == 0 || (!col && !val)) return PLX_OK;
    k_move_entries<<<grid_for(o.nnz), kThreads, 0, ctx->stream>>>(o.rows, o.nnz, o.bptr, o.row_order, o.rowptr,
                                                                  col ? o.col : nullptr, val ? o.val : nullptr, col, val, 0);
    PLX_HIP(ctx, hipGetLastError());
    return PLX_OK;
}

}  // namespace plx

using namespace plx;

extern "C" {

plx_status plx_build_csr(plx_ctx* ctx, int64_t n, int64_t n_edges, const int64_t* src, const int64_t* dst,
                         const int64_t* perm_r, const int64_t* perm_c, plx_csr** out) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!out) return fail(ctx, PLX_ERR_INVALID, "out is NULL");
    *out = nullptr;
    if (n < 0 || n_edges < 0) return fail(ctx, PLX_ERR_INVALID, "negative size");
    if (n_edges > 0 && (!src || !dst)) return fail(ctx, PLX_ERR_INVALID, "src or dst is NULL");
    if (n >= (int64_t(1) << 31)) return fail(ctx, PLX_ERR_UNSUPPORTED, "n = %lld needs 64-bit column ids", (long long)n);
    const int64_t count = 2 * n_edges + n;
    if (count >= (int64_t(1) << 31)) return fail(ctx, PLX_ERR_UNSUPPORTED, "more than 2^31-1 candidate entries");
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");
    PLX_HIP(ctx, hipSetDevice(ctx->device));

    plx_csr* h = new (std::nothrow) plx_csr();
    if (!h) return fail(ctx, PLX_ERR_OOM, "host allocation failed");
    auto bail = [&](plx_status s) { plx_csr_destroy(ctx, h); return s; };
    plx_status st = [&]() -> plx_status {
        TempPool pool(ctx);
        hipStream_t s = ctx->stream;
        int* flags = pool.get<int>(1);
        if (!flags) return PLX_ERR_OOM;
        PLX_HIP(ctx, hipMemsetAsync(flags, 0, sizeof(int), s));
        if (n_edges > 0) k_check_ids<<<grid_for(n_edges), kThreads, 0, s>>>(n, n_edges, src, dst, flags);
        {
            TempPool hp(ctx);
            for (const int64_t* p : {perm_r, perm_c}) {
                if (!p || n == 0) continue;
                int* hits = hp.get<int>(n);
                if (!hits) return PLX_ERR_OOM;
                PLX_HIP(ctx, hipMemsetAsync(hits, 0, sizeof(int) * n, s));
                k_mark_perm<<<grid_for(n), kThreads, 0, s>>>(n, p, hits, flags);
                k_check_hits<<<grid_for(n), kThreads, 0, s>>>(n, hits, flags);
            }
            int hf = 0;
            PLX_HIP(ctx, hipMemcpyAsync(&hf, flags, sizeof(int), hipMemcpyDeviceToHost, s));
            PLX_HIP(ctx, hipStreamSynchronize(s));
            if (hf & kFlagBadId) return fail(ctx, PLX_ERR_INVALID, "edge list holds a node id outside [0, n)");
            if (hf & kFlagBadPerm) return fail(ctx, PLX_ERR_INVALID, "a permutation is not a bijection on [0, n)");
        }
        Orient& f = h->o[0];
        f.rows = f.cols = n;
        f.rowptr = static_cast<int64_t*>(dev_alloc(ctx, sizeof(int64_t) * (n + 1)));
        h->deg = static_cast<int64_t*>(dev_alloc(ctx, sizeof(int64_t) * std::max<int64_t>(1, n)));
        h->n_deg = n;
        if (!f.rowptr || !h->deg) return PLX_ERR_OOM;
        int32_t* row = nullptr;
        if (n == 0) {
            PLX_HIP(ctx, hipMemsetAsync(f.rowptr, 0, sizeof(int64_t), s));
            f.col = static_cast<int32_t*>(dev_alloc(ctx, 4));
            f.val = static_cast<float*>(dev_alloc(ctx, 4));
            if (!f.col || !f.val) return PLX_ERR_OOM;
        } else {
            const uint64_t sentinel = (uint64_t)n * (uint64_t)n;
            uint64_t* keys = pool.get<uint64_t>(count);
            uint64_t* sorted = pool.get<uint64_t>(count);
            if (!keys || !sorted) return PLX_ERR_OOM;
            k_make_keys<<<grid_for(n_edges + n), kThreads, 0, s>>>(n, n_edges, src, dst, perm_r, perm_c, keys, sentinel);
            {
                int bits = bit_length(sentinel);
                size_t bytes = 0;
                PLX_HIP(ctx, rocprim::radix_sort_keys(nullptr, bytes, keys, sorted, (size_t)count, 0, bits, s));
                void* tmp = pool.get<char>(bytes);
                if (!tmp) return PLX_ERR_OOM;
                PLX_HIP(ctx, rocprim::radix_sort_keys(tmp, bytes, keys, sorted, (size_t)count, 0, bits, s));
            }
            uint32_t* flag = pool.get<uint32_t>(count + 1);
            uint32_t* pos = pool.get<uint32_t>(count + 1);
            if (!flag || !pos) return PLX_ERR_OOM;
            PLX_HIP(ctx, hipMemsetAsync(flag + count, 0, sizeof(uint32_t), s));
            k_flag_unique<<<grid_for(count), kThreads, 0, s>>>(count, sorted, sentinel, flag);
            PLX_TRY(scan_exclusive<uint32_t>(ctx, pool, flag, pos, (size_t)count + 1));
            uint32_t nnz32 = 0;
            PLX_HIP(ctx, hipMemcpyAsync(&nnz32, pos + count, sizeof(uint32_t), hipMemcpyDeviceToHost, s));
            PLX_HIP(ctx, hipStreamSynchronize(s));
            f.nnz = nnz32;
            f.col = static_cast<int32_t*>(dev_alloc(ctx, sizeof(int32_t) * f.nnz));
            f.val = static_cast<float*>(dev_alloc(ctx, sizeof(float) * f.nnz));
            row = pool.get<int32_t>(f.nnz);
            unsigned int* rowcount = pool.get<unsigned int>(n + 1);
            int64_t* deg_c = pool.get<int64_t>(n);
            if (!f.col || !f.val || !row || !rowcount || !deg_c) return PLX_ERR_OOM;
            PLX_HIP(ctx, hipMemsetAsync(rowcount, 0, sizeof(unsigned int) * (n + 1), s));
            k_scatter_unique<<<grid_for(count), kThreads, 0, s>>>(count, sorted, flag, pos, (uint64_t)n, row, f.col, rowcount);
            PLX_TRY(counts_to_rowptr(ctx, pool, rowcount, n, f.rowptr));
            k_degrees<<<grid_for(n), kThreads, 0, s>>>(n, f.rowptr, perm_r, perm_c, h->deg, deg_c);
            k_values<<<grid_for(f.nnz), kThreads, 0, s>>>(f.nnz, row, f.col, f.rowptr, deg_c, f.val);
            PLX_HIP(ctx, hipGetLastError());
            PLX_TRY(transpose_orient(ctx, f, row, h->o[1]));
        }
        if (n == 0) {
            Orient& b = h->o[1];
            b.rowptr = static_cast<int64_t*>(dev_alloc(ctx, sizeof(int64_t)));
            b.col = static_cast<int32_t*>(dev_alloc(ctx, 4));
            b.val = static_cast<float*>(dev_alloc(ctx, 4));
            if (!b.rowptr || !b.col || !b.val) return PLX_ERR_OOM;
            PLX_HIP(ctx, hipMemsetAsync(b.rowptr, 0, sizeof(int64_t), s));
        }
        h->o[1].tag = 1;
        PLX_TRY(build_bins(ctx, h->o[0]));
        PLX_TRY(build_bins(ctx, h->o[1]));
        PLX_HIP(ctx, hipStreamSynchronize(s));
        PLX_HIP(ctx, hipGetLastError());
        return PLX_OK;
    }();
    if (st != PLX_OK) return bail(st);
    *out = h;
    return PLX_OK;
}

plx_status plx_csr_import(plx_ctx* ctx, int64_t m, int64_t k, int64_t nnz, const int64_t* rowptr, const int32_t* col,
                          const float* val, plx_csr** out) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!out) return fail(ctx, PLX_ERR_INVALID, "out is NULL");
    *out = nullptr;
    if (m < 0 || k < 0 || nnz < 0) return fail(ctx, PLX_ERR_INVALID, "negative size");
    if (!rowptr || (nnz > 0 && (!col || !val))) return fail(ctx, PLX_ERR_INVALID, "rowptr, col or val is NULL");
    if (m >= (int64_t(1) << 31) || k >= (int64_t(1) << 31) || nnz >= (int64_t(1) << 31))
        return fail(ctx, PLX_ERR_UNSUPPORTED, "a dimension or the entry count needs more than 31 bits");
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");
    PLX_HIP(ctx, hipSetDevice(ctx->device));

    plx_csr* h = new (std::nothrow) plx_csr();
    if (!h) return fail(ctx, PLX_ERR_OOM, "host allocation failed");
    plx_status st = [&]() -> plx_status {
        TempPool pool(ctx);
        hipStream_t s = ctx->stream;
        Orient& f = h->o[0];
        f.rows = m; f.cols = k; f.nnz = nnz;
        f.rowptr = static_cast<int64_t*>(dev_alloc(ctx, sizeof(int64_t) * (m + 1)));
        f.col = static_cast<int32_t*>(dev_alloc(ctx, sizeof(int32_t) * std::max<int64_t>(1, nnz)));
        f.val = static_cast<float*>(dev_alloc(ctx, sizeof(float) * std::max<int64_t>(1, nnz)));
        int* flags = pool.get<int>(1);
        int32_t* row = pool.get<int32_t>(nnz);
        if (!f.rowptr || !f.col || !f.val || !flags || !row) return PLX_ERR_OOM;
        PLX_HIP(ctx, hipMemsetAsync(flags, 0, sizeof(int), s));
        k_check_rowptr<<<grid_for(m + 1), kThreads, 0, s>>>(m, nnz, rowptr, flags);
        int hf = 0;
        PLX_HIP(ctx, hipMemcpyAsync(&hf, flags, sizeof(int), hipMemcpyDeviceToHost, s));
        PLX_HIP(ctx, hipStreamSynchronize(s));
        if (hf) return fail(ctx, PLX_ERR_INVALID, "rowptr is not a non-decreasing array from 0 to nnz");
        PLX_HIP(ctx, hipMemcpyAsync(f.rowptr, rowptr, sizeof(int64_t) * (m + 1), hipMemcpyDeviceToDevice, s));
        if (nnz > 0) {
            PLX_HIP(ctx, hipMemcpyAsync(f.col, col, sizeof(int32_t) * nnz, hipMemcpyDeviceToDevice, s));
            PLX_HIP(ctx, hipMemcpyAsync(f.val, val, sizeof(float) * nnz, hipMemcpyDeviceToDevice, s));
            k_expand_rows<<<grid_for(nnz), kThreads, 0, s>>>(m, nnz, f.rowptr, row);
            k_check_cols<<<grid_for(nnz), kThreads, 0, s>>>(nnz, k, row, f.col, flags);
            PLX_HIP(ctx, hipMemcpyAsync(&hf, flags, sizeof(int), hipMemcpyDeviceToHost, s));
            PLX_HIP(ctx, hipStreamSynchronize(s));
            if (hf) return fail(ctx, PLX_ERR_INVALID, "column ids must lie in [0, k) and ascend strictly inside a row");
        }
        PLX_TRY(transpose_orient(ctx, f, row, h->o[1]));
        h->o[1].tag = 1;
        PLX_TRY(build_bins(ctx, h->o[0]));
        PLX_TRY(build_bins(ctx, h->o[1]));
        PLX_HIP(ctx, hipStreamSynchronize(s));
        PLX_HIP(ctx, hipGetLastError());
        return PLX_OK;
    }();
    if (st != PLX_OK) { plx_csr_destroy(ctx, h); return st; }
    *out = h;
    return PLX_OK;
}

plx_status plx_csr_set_row_blocks(plx_ctx* ctx, plx_csr* csr, int n_blocks) {
    if (!ctx) return PLX_ERR_INVALID;
    if (!csr) return fail(ctx, PLX_ERR_INVALID, "csr is NULL");
    if (n_blocks < 1 || n_blocks > 64) return fail(ctx, PLX_ERR_INVALID, "n_blocks must be between 1 and 64");
    if (ctx->dry) return fail(ctx, PLX_ERR_DEVICE, "validate-only context");
    PLX_HIP(ctx, hipSetDevice(ctx->device));
    for (int t = 0; t < 2; ++t) {
        Orient& o = csr->o[t];
        if (o.n_blocks == n_blocks) continue;
        PLX_TRY(unbin(ctx, o));
        PLX_TRY(build_bins(ctx, o, n_blocks));
    }
    PLX_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return PLX_OK;
}

}  // extern "C"
