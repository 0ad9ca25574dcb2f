// Sparse x dense product Y = A X for a CSR orientation (paper Eq. 2.1; with the transposed
// orientation also Eq. 2.7).  The product is bound by the gather of dense rows of X from HBM:
// every stored entry fetches one row of X (the double permutation of Sec. 5.1 leaves no
// locality between neighbouring entries), so the kernels are organised around wide, fully used
// memory transactions and many independent gathers in flight:
//
//  * a dense row of d elements is covered by G = 2^ceil(log2(ceil(d / VW))) lanes, each holding
//    VW consecutive elements (one 128-bit load when the layout allows it);
//  * rows are binned by length class (set-up time).  Short rows (< 256 entries): one G-lane group
//    per row, 64/G rows per wavefront, no cross-lane traffic.  Longer rows are cut into segments
//    at the boundaries of a few equal column windows (and to a maximum length); one wavefront per
//    segment, its 64/G groups stride over the entries and are combined by a butterfly across
//    groups; the partial sums of a row are added in segment order by a second kernel (no
//    floating-point atomics => bit-reproducible).  Segments are launched window by window: a
//    row's entries are sorted by column, so the wavefronts running at any moment gather from one
//    band of X, which is read from HBM once and then hits in the Infinity Cache / L2.  With the
//    windows switched off, rows below 4096 entries take a wavefront-per-row kernel instead;
//  * the entry loop is unrolled U-fold with all column/value loads issued before the U gathers,
//    so a lane keeps U independent gathers in flight.
#include "plx_internal.h"

#include <algorithm>
#include <mutex>
#include <type_traits>

namespace plx {
namespace {

typedef uint16_t bf16_t;
typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {   // round to nearest even
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <int BYTES> struct Raw;
template <> struct Raw<2> { typedef uint16_t type; };
template <> struct Raw<4> { typedef uint32_t type; };
template <> struct Raw<8> { typedef uint2 type; };
template <> struct Raw<16> { typedef uint4 type; };

// Output rows are written once and not read again by this kernel: non-temporal stores leave the
// cache to the gathered operand rows (measured: 2-9 % off the short-row kernel; non-temporal
// LOADS of the CSR arrays were measured slower and are not used).
template <int BYTES> struct Ext;
template <> struct Ext<2> { typedef uint16_t type; };
template <> struct Ext<4> { typedef uint32_t type; };
template <> struct Ext<8> { typedef uint32_t type __attribute__((ext_vector_type(2))); };
template <> struct Ext<16> { typedef uint32_t type __attribute__((ext_vector_type(4))); };

// Gathered rows wait in registers as they were loaded (a bf16 row of 8 is 4 registers, not 8 floats): one transaction
// now, widened and accumulated when the row is used.
template <typename T, int VW> struct RowRegs { typename Raw<sizeof(T) * VW>::type raw; };
template <typename T, int VW>
__device__ __forceinline__ RowRegs<T, VW> load_row(const T* p) {
    RowRegs<T, VW> r;
    r.raw = *reinterpret_cast<const typename Raw<sizeof(T) * VW>::type*>(p);
    return r;
}
template <typename T, int VW>
__device__ __forceinline__ RowRegs<T, VW> zero_row() {
    RowRegs<T, VW> r;
    union { typename Raw<sizeof(T) * VW>::type raw; T e[VW]; } u;
#pragma unroll
    for (int i = 0; i < VW; ++i) u.e[i] = T(0);
    r.raw = u.raw;
    return r;
}
template <typename T, int VW>
__device__ __forceinline__ void fma_row(float v, const RowRegs<T, VW>& r, float (&acc)[VW]) {
    union { typename Raw<sizeof(T) * VW>::type raw; T e[VW]; } u;
    u.raw = r.raw;
#pragma unroll
    for (int i = 0; i < VW; ++i) {
        if constexpr (sizeof(T) == 4) acc[i] = fmaf(v, u.e[i], acc[i]);
        else acc[i] = fmaf(v, bf16_to_f32(u.e[i]), acc[i]);
    }
}

template <typename T> __device__ __forceinline__ T narrow(float f) {
    if constexpr (sizeof(T) == 4) return f;
    else return f32_to_bf16(f);
}

// store the first `valid` of VW elements (one transaction when all are valid)
template <typename T, int VW>
__device__ __forceinline__ void store_vec(T* p, const float (&r)[VW], int valid) {
    typedef typename Raw<sizeof(T) * VW>::type raw_t;
    if (valid >= VW) {
        union { raw_t raw; T e[VW]; } u;
#pragma unroll
        for (int i = 0; i < VW; ++i) u.e[i] = narrow<T>(r[i]);
        typedef typename Ext<sizeof(T) * VW>::type ext_t;
        union { raw_t raw; ext_t ext; } w;
        w.raw = u.raw;
        __builtin_nontemporal_store(w.ext, reinterpret_cast<ext_t*>(p));
    } else {
#pragma unroll
        for (int i = 0; i < VW; ++i)
            if (i < valid) p[i] = narrow<T>(r[i]);
    }
}

// Where a finished output row goes: Y (plain) and / or Yact (after ReLU, Eq. 2.3); either may be NULL.
template <typename T> struct Out {
    T* y; int64_t ldy;
    T* ya; int64_t ldya;
};

template <typename T, int VW>
__device__ __forceinline__ void emit(const Out<T>& o, int64_t row, int c0, float (&acc)[VW], int valid) {
    if (o.y) store_vec<T, VW>(o.y + row * o.ldy + c0, acc, valid);
    if (o.ya) {
#pragma unroll
        for (int i = 0; i < VW; ++i) acc[i] = acc[i] > 0.f ? acc[i] : 0.f;
        store_vec<T, VW>(o.ya + row * o.ldya + c0, acc, valid);
    }
}

#ifndef PLX_SPMM_UNROLL
#define PLX_SPMM_UNROLL 8
#endif
#ifndef PLX_SPMM_UNROLL_WIDE
#define PLX_SPMM_UNROLL_WIDE 4
#endif
// Gathers a lane keeps in flight per trip.  Their rows wait in registers as VW floats each: 8 x 4 for fp32 and 4 x 8 for
// bf16 are the same 32 registers (8 x 8 leaves a bf16 kernel with too few resident wavefronts: measured 7-25 % slower on
// the segment kernels and on the staged short-row kernel of every workload).
template <int VW> constexpr int gathers_per_trip() { return VW > 4 ? PLX_SPMM_UNROLL_WIDE : PLX_SPMM_UNROLL; }

// acc += sum over entries e = first, first + stride, ... < hi of val[e] * X[col[e], c0 .. c0+VW), kUnroll gathers per trip
template <typename T, int VW, int kUnroll = gathers_per_trip<VW>()>
__device__ __forceinline__ void gather_accumulate(int64_t first, int64_t hi, int64_t stride,
                                                  const int32_t* __restrict__ col, const float* __restrict__ val,
                                                  const T* __restrict__ xb, int64_t ldx, float (&acc)[VW]) {
    int64_t e = first;
    for (; e + (kUnroll - 1) * stride < hi; e += kUnroll * stride) {
        int32_t c[kUnroll];
        float v[kUnroll];
#pragma unroll
        for (int t = 0; t < kUnroll; ++t) { c[t] = col[e + t * stride]; v[t] = val[e + t * stride]; }
        RowRegs<T, VW> x[kUnroll];
#pragma unroll
        for (int t = 0; t < kUnroll; ++t) x[t] = load_row<T, VW>(xb + (int64_t)c[t] * ldx);
#pragma unroll
        for (int t = 0; t < kUnroll; ++t) fma_row<T, VW>(v[t], x[t], acc);
    }
    if (e < hi) {
        // what is left is fewer than kUnroll entries: one more trip with the missing ones masked off, so that the
        // remaining gathers are in flight together too (a segment of a long row is often shorter than one full trip)
        int32_t c[kUnroll];
        float v[kUnroll];
        bool ok[kUnroll];
#pragma unroll
        for (int t = 0; t < kUnroll; ++t) {
            const int64_t idx = e + t * stride;
            ok[t] = idx < hi;
            c[t] = ok[t] ? col[idx] : 0;
            v[t] = ok[t] ? val[idx] : 0.f;
        }
        RowRegs<T, VW> x[kUnroll];
#pragma unroll
        for (int t = 0; t < kUnroll; ++t) x[t] = ok[t] ? load_row<T, VW>(xb + (int64_t)c[t] * ldx) : zero_row<T, VW>();
#pragma unroll
        for (int t = 0; t < kUnroll; ++t) fma_row<T, VW>(v[t], x[t], acc);
    }
}

// Tuning switches of the short-row kernel (compile time).
#ifndef PLX_SUB_STAGED
#define PLX_SUB_STAGED 1      // 1: a group loads its (column, value) pairs once, coalesced, and shares them by lane shuffles
#endif
#ifndef PLX_SUB_PERSIST
#define PLX_SUB_PERSIST 64    // N > 0: grid of N workgroups per CU, every group of lanes walks several rows (measured: 16 < 32 < 64)
#endif

// Same sum as gather_accumulate for a contiguous entry range, but the G lanes of a group fetch
// up to CH entries with one coalesced load each for columns and values and pass them round by
// shuffles, instead of every lane loading every entry.  All lanes of the group must call it.
template <typename T, int G, int VW>
__device__ __forceinline__ void gather_staged(int64_t lo, int64_t hi, const int32_t* __restrict__ col,
                                              const float* __restrict__ val, const T* __restrict__ xb, int64_t ldx,
                                              bool active, int lane, float (&acc)[VW]) {
    constexpr int CH = G < gathers_per_trip<VW>() ? G : gathers_per_trip<VW>();
    const int j = lane % G, gbase = lane - j;
    for (int64_t e = lo; e < hi; e += CH) {
        const int n = (hi - e) < CH ? (int)(hi - e) : CH;
        int32_t cj = 0;
        float vj = 0.f;
        if (j < n) { cj = col[e + j]; vj = val[e + j]; }
        int32_t c[CH];
        float v[CH];
#pragma unroll
        for (int t = 0; t < CH; ++t) { c[t] = __shfl(cj, gbase + t, kWave); v[t] = __shfl(vj, gbase + t, kWave); }
        RowRegs<T, VW> x[CH];
#pragma unroll
        for (int t = 0; t < CH; ++t) x[t] = (active && t < n) ? load_row<T, VW>(xb + (int64_t)c[t] * ldx) : zero_row<T, VW>();
#pragma unroll
        for (int t = 0; t < CH; ++t) fma_row<T, VW>(v[t], x[t], acc);
    }
}

// Short rows: one group of G lanes per row, 64/G rows per wavefront.
template <typename T, int G, int VW>
__global__ __launch_bounds__(256) void k_spmm_subwave(const int32_t* __restrict__ row_order, int64_t count,
                                                      const int32_t* __restrict__ bptr,
                                                      const int32_t* __restrict__ col, const float* __restrict__ val,
                                                      const T* __restrict__ X, int64_t ldx, Out<T> out, int d) {
    constexpr int R = kWave / G;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    const int c0 = (lane % G) * VW;
    const bool active = c0 < d;
#if PLX_SUB_PERSIST
    const int64_t stride = (int64_t)gridDim.x * (blockDim.x / kWave) * R;
#else
    const int64_t stride = count;   // one row per group
#endif
    for (int64_t slot = wave * R + lane / G; slot < count; slot += stride) {
        const int32_t row = row_order[slot];
        const int64_t lo = bptr[slot], hi = bptr[slot + 1];
        float acc[VW];
#pragma unroll
        for (int i = 0; i < VW; ++i) acc[i] = 0.f;
#if PLX_SUB_STAGED
        if constexpr (G >= 8) gather_staged<T, G, VW>(lo, hi, col, val, X + c0, ldx, active, lane, acc);
        else if (active) gather_accumulate<T, VW, PLX_SPMM_UNROLL>(lo, hi, 1, col, val, X + c0, ldx, acc);   // narrow rows (G < 8): 8 per trip measured better for either type
#else
        if (active) gather_accumulate<T, VW>(lo, hi, 1, col, val, X + c0, ldx, acc);
#endif
        if (active) emit<T, VW>(out, row, c0, acc, d - c0);
    }
}

// butterfly sum across the 64/G groups of a wavefront; every lane ends with the total
template <int G, int VW>
__device__ __forceinline__ void reduce_groups(float (&acc)[VW]) {
#pragma unroll
    for (int off = G; off < kWave; off <<= 1)
#pragma unroll
        for (int i = 0; i < VW; ++i) acc[i] += __shfl_xor(acc[i], off, kWave);
}

// Medium rows: one wavefront per row.
template <typename T, int G, int VW>
__global__ __launch_bounds__(256) void k_spmm_wave(const int32_t* __restrict__ rows, int64_t count,
                                                   const int32_t* __restrict__ bptr,
                                                   const int32_t* __restrict__ col, const float* __restrict__ val,
                                                   const T* __restrict__ X, int64_t ldx, Out<T> out, int d) {
    constexpr int NG = kWave / G;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t slot = (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (slot >= count) return;                       // uniform per wavefront
    const int g = lane / G, c0 = (lane % G) * VW;
    const bool active = c0 < d;
    const int32_t row = rows[slot];
    const int64_t lo = bptr[slot], hi = bptr[slot + 1];
    float acc[VW];
#pragma unroll
    for (int i = 0; i < VW; ++i) acc[i] = 0.f;
    if (active) gather_accumulate<T, VW>(lo + g, hi, NG, col, val, X + c0, ldx, acc);
    reduce_groups<G, VW>(acc);
    if (g == 0 && active) emit<T, VW>(out, row, c0, acc, d - c0);
}

// Long rows, stage 1: one wavefront per segment, fp32 partial sums to part[seg][G*VW].  The segment's record sits at a
// wave-uniform address (scalar loads: the chain record -> columns -> operand rows has one vector-memory step less).
template <typename T, int G, int VW>
__global__ __launch_bounds__(256) void k_spmm_segment(int64_t n_seg, const int4* __restrict__ desc,
                                                      const int32_t* __restrict__ col, const float* __restrict__ val,
                                                      const T* __restrict__ X, int64_t ldx, float* __restrict__ part,
                                                      int d) {
    constexpr int NG = kWave / G;
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int64_t pos = (int64_t)blockIdx.x * (blockDim.x / kWave) + wv;
    if (pos >= n_seg) return;
    const int4 rec = desc[pos];                      // launch order (column window by window)
    const int64_t seg = rec.z;
    const int g = lane / G, c0 = (lane % G) * VW;
    const bool active = c0 < d;
    const int64_t lo = rec.x, hi = lo + rec.y;
    float acc[VW];
#pragma unroll
    for (int i = 0; i < VW; ++i) acc[i] = 0.f;
    if (active) gather_accumulate<T, VW>(lo + g, hi, NG, col, val, X + c0, ldx, acc);
    reduce_groups<G, VW>(acc);
    if (g == 0) {
        float* p = part + seg * (G * VW) + c0;
#pragma unroll
        for (int i = 0; i < VW; ++i) p[i] = acc[i];
    }
}

// Long rows, stage 2: Y[row] = sum of the row's segment partials, in segment order.
template <typename T>
__global__ __launch_bounds__(256) void k_spmm_combine(int64_t n_long, const int32_t* __restrict__ long_row,
                                                      const int32_t* __restrict__ seg0, const float* __restrict__ part,
                                                      int ldp, Out<T> out, int d) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t q = idx / d;
    const int j = (int)(idx % d);
    if (q >= n_long) return;
    float s = 0.f;
    for (int32_t k = seg0[q]; k < seg0[q + 1]; ++k) s += part[(int64_t)k * ldp + j];
    const int64_t row = long_row[q];
    if (out.y) out.y[row * out.ldy + j] = narrow<T>(s);
    if (out.ya) out.ya[row * out.ldya + j] = narrow<T>(s > 0.f ? s : 0.f);
}

// ---- aggregation with the combination in its epilogue (Eq. 2.1 -> 2.2 -> 2.3 in one pass over the short rows) -------
// The short-row kernel above, for fp32 rows of 17..32 elements (G = 8 lanes per row, 8 rows per wavefront and trip),
// that keeps the aggregated rows on chip: four trips fill a wave-private 32 x 32 tile of H = A X in LDS (H is still
// written out: Eq. 2.5 reads it in the backward pass), and the tile is multiplied by W[din x dout] (in LDS, once per
// workgroup) with v_mfma_f32_32x32x2_f32 -- lane l: a = H[row l%32][k = 2s + l/32], b = W[2s + l/32][32 nb + l%32],
// acc[r] = result[row 8(r/4) + 4(l/32) + r%4][32 nb + l%32] -- and leaves as Q and / or ReLU(Q) and / or its sign bits
// for the rows' ids.  What it saves is the combination's re-read of H; what it costs is registers and LDS in a kernel
// that lives on the number of gathers in flight.
constexpr int kEpiRows = 32, kEpiHP = 33;

template <int TNB>
struct EpiLds {
    static constexpr int WP = 32 * TNB + 4;
    static constexpr size_t floats = 32 * WP + (256 / kWave) * kEpiRows * kEpiHP;
    static constexpr size_t bytes = floats * sizeof(float) + (256 / kWave) * kEpiRows * sizeof(int) +
                                    (256 / kWave) * kEpiRows * 4 * sizeof(uint32_t);
};

template <int TNB>
__device__ __forceinline__ void epi_load_weights(float* Wl, const float* __restrict__ W, int64_t ldw, int din, int dout) {
    constexpr int WP = EpiLds<TNB>::WP;
    for (int i = threadIdx.x; i < 32 * 32 * TNB; i += 256) {
        const int k = i / (32 * TNB), n = i % (32 * TNB);
        Wl[k * WP + n] = (k < din && n < dout) ? W[(int64_t)k * ldw + n] : 0.f;
    }
}

// one wavefront: result rows of its 32 x 32 tile Ht (row ids in rid, -1 = no row) times Wl, written out
template <int TNB>
__device__ __forceinline__ void epi_tile(const float* Ht, const int* rid, uint32_t* wb, const float* Wl, int din, int dout,
                                         float* __restrict__ C, int64_t ldc, float* __restrict__ F, int64_t ldf,
                                         uint32_t* __restrict__ bits, int64_t ldbits, int lane) {
    constexpr int WP = EpiLds<TNB>::WP;
    const int l32 = lane & 31, lh = lane >> 5;
    const int ks = (din + 1) / 2;
    int rows[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) rows[r] = rid[8 * (r / 4) + 4 * lh + (r % 4)];
#pragma unroll
    for (int nb = 0; nb < TNB; ++nb) {
        if (32 * nb >= dout) break;                                      // uniform
        floatx16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll 4
        for (int s2 = 0; s2 < ks; ++s2)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(Ht[l32 * kEpiHP + 2 * s2 + lh], Wl[(2 * s2 + lh) * WP + 32 * nb + l32], acc, 0, 0, 0);
        const int n = 32 * nb + l32;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float v = acc[r];
            if (rows[r] >= 0 && n < dout) {
                if (C) __builtin_nontemporal_store(v, C + (int64_t)rows[r] * ldc + n);
                if (F) __builtin_nontemporal_store(v > 0.f ? v : 0.f, F + (int64_t)rows[r] * ldf + n);
            }
            if (bits) {                                                   // 32 columns of two rows per ballot; columns >= dout give 0
                const unsigned long long b = __ballot(v > 0.f && n < dout);
                if (lane == 0) {
                    const int t0 = 8 * (r / 4) + (r % 4);
                    wb[t0 * 4 + nb] = (uint32_t)b;
                    wb[(t0 + 4) * 4 + nb] = (uint32_t)(b >> 32);
                }
            }
        }
    }
    if (bits) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const int nw = (dout + 31) >> 5;
        if (lane < kEpiRows && rid[lane] >= 0) {
            uint32_t* dst = bits + (int64_t)rid[lane] * ldbits;
            for (int j = 0; j < nw; ++j) dst[j] = wb[lane * 4 + j];
        }
    }
}

template <int TNB>
__global__ __launch_bounds__(256) void k_spmm_subwave_combine(const int32_t* __restrict__ row_order, int64_t count,
                                                              const int32_t* __restrict__ bptr, const int32_t* __restrict__ col,
                                                              const float* __restrict__ val, const float* __restrict__ X, int64_t ldx,
                                                              float* __restrict__ S, int64_t lds_, const float* __restrict__ W,
                                                              int64_t ldw, int din, int dout, float* __restrict__ C, int64_t ldc,
                                                              float* __restrict__ F, int64_t ldf, uint32_t* __restrict__ bits,
                                                              int64_t ldbits) {
    constexpr int G = 8, VW = 4, R = kWave / G;
    extern __shared__ __align__(16) float epi_smem[];
    float* Wl = epi_smem;
    const int lane = threadIdx.x & (kWave - 1), wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    float* Ht = Wl + 32 * EpiLds<TNB>::WP + wv * (kEpiRows * kEpiHP);
    int* rid = reinterpret_cast<int*>(Wl + EpiLds<TNB>::floats) + wv * kEpiRows;
    uint32_t* wb = reinterpret_cast<uint32_t*>(reinterpret_cast<int*>(Wl + EpiLds<TNB>::floats) + (256 / kWave) * kEpiRows) + wv * kEpiRows * 4;
    epi_load_weights<TNB>(Wl, W, ldw, din, dout);
    __syncthreads();
    const int c0 = (lane % G) * VW;
    const bool active = c0 < din;
    const int64_t stride = (int64_t)gridDim.x * (blockDim.x / kWave) * R;
    int filled = 0;                                                      // trips in the tile so far (uniform)
    for (int64_t base = ((int64_t)blockIdx.x * (blockDim.x / kWave) + wv) * R; base < count; base += stride) {
        const int64_t slot = base + lane / G;
        const bool valid = slot < count;
        const int32_t row = valid ? row_order[slot] : -1;
        const int64_t lo = valid ? bptr[slot] : 0, hi = valid ? bptr[slot + 1] : 0;
        float acc[VW];
#pragma unroll
        for (int i = 0; i < VW; ++i) acc[i] = 0.f;
        gather_staged<float, G, VW>(lo, hi, col, val, X + c0, ldx, active, lane, acc);
        if (valid && active) store_vec<float, VW>(S + (int64_t)row * lds_ + c0, acc, din - c0);      // H itself (Eq. 2.1)
        const int tr = filled * R + lane / G;
#pragma unroll
        for (int i = 0; i < VW; ++i) Ht[tr * kEpiHP + c0 + i] = c0 + i < din ? acc[i] : 0.f;   // beyond din a vector holds the row's padding
        if (lane % G == 0) rid[tr] = row;
        if (++filled == kEpiRows / R) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            epi_tile<TNB>(Ht, rid, wb, Wl, din, dout, C, ldc, F, ldf, bits, ldbits, lane);
            __builtin_amdgcn_wave_barrier();
            filled = 0;
        }
    }
    if (filled > 0) {                                                    // a last, partial tile: the missing rows have no id
        for (int t = filled * R + lane; t < kEpiRows; t += kWave) rid[t] = -1;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        epi_tile<TNB>(Ht, rid, wb, Wl, din, dout, C, ldc, F, ldf, bits, ldbits, lane);
    }
}

// The same epilogue for listed rows whose H is already in memory (the rows summed from segments): one wavefront per
// 32 rows of the list.
template <int TNB>
__global__ __launch_bounds__(256) void k_rows_combine(int64_t n_rows, const int32_t* __restrict__ list, const float* __restrict__ S,
                                                      int64_t lds_, const float* __restrict__ W, int64_t ldw, int din, int dout,
                                                      float* __restrict__ C, int64_t ldc, float* __restrict__ F, int64_t ldf,
                                                      uint32_t* __restrict__ bits, int64_t ldbits) {
    extern __shared__ __align__(16) float epi_smem[];
    float* Wl = epi_smem;
    const int lane = threadIdx.x & (kWave - 1), wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    float* Ht = Wl + 32 * EpiLds<TNB>::WP + wv * (kEpiRows * kEpiHP);
    int* rid = reinterpret_cast<int*>(Wl + EpiLds<TNB>::floats) + wv * kEpiRows;
    uint32_t* wb = reinterpret_cast<uint32_t*>(reinterpret_cast<int*>(Wl + EpiLds<TNB>::floats) + (256 / kWave) * kEpiRows) + wv * kEpiRows * 4;
    epi_load_weights<TNB>(Wl, W, ldw, din, dout);
    __syncthreads();
    const int64_t q0 = ((int64_t)blockIdx.x * (blockDim.x / kWave) + wv) * kEpiRows;
    if (q0 >= n_rows) return;                                            // uniform per wavefront
    if (lane < kEpiRows) rid[lane] = q0 + lane < n_rows ? list[q0 + lane] : -1;
    for (int i = lane; i < kEpiRows * 32; i += kWave) {
        const int t = i / 32, k = i % 32;
        const int64_t q = q0 + t;
        Ht[t * kEpiHP + k] = (q < n_rows && k < din) ? S[(int64_t)list[q] * lds_ + k] : 0.f;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    epi_tile<TNB>(Ht, rid, wb, Wl, din, dout, C, ldc, F, ldf, bits, ldbits, lane);
}

// Where the partial sums of the segments go: the handle's own buffer (kPartFloats floats per segment, sized when the
// handle was built), or memory the caller of launch_spmm brought (`given`, the allocation-free entry point: used as it
// is, and nothing is timed there because the timer creates events).  Either way a product allocates nothing.
struct Partials {
    float* given = nullptr;
    size_t bytes = 0;
};

constexpr int WPB = 256 / kWave;   // wavefronts per block

// Rows below the segment threshold: one group of lanes per row (and one wavefront per row where the column windows are off).
template <typename T, int G, int VW>
plx_status run_short(plx_ctx* ctx, const Orient& o, int blk, const T* X, int64_t ldx, Out<T> out, int d, bool timed) {
    hipStream_t s = ctx->stream;
    const int64_t s0 = o.off(blk, 0);                                  // first slot of this row block
    const int64_t n_sub = o.off(blk, kSubwaveMaxClass + 1) - s0;
    const int64_t n_wave = o.off(blk, o.long_class) - s0 - n_sub;      // none when every such row goes through segments
    char label[64];
    if (timed) snprintf(label, sizeof label, "<%s,G%d,VW%d,d%d>[%s]", sizeof(T) == 4 ? "f32" : "bf16", G, VW, d, o.tag ? "At" : "A");
    if (n_sub > 0) {
        KernelTimer kt(ctx, timed ? std::string("spmm_subwave") + label : std::string(), timed);
        constexpr int R = kWave / G;
        int64_t blocks = ceil_div(ceil_div(n_sub, R), WPB);
#if PLX_SUB_PERSIST
        // A persistent grid evens out rows of unequal length (a power-law bin holds rows of 1 to 255 entries).  Where
        // practically every row fits one trip of 8 entries (a road-like graph: fewer than 1 in 1000 rows is longer) there
        // is nothing to even out and one row per group of lanes is faster (road network: -5 to -12 % on its four
        // short-row launches; the shard's bins, with 10 % longer rows, lose 15 - 24 % that way and keep the persistent grid).
        const int64_t n_longer = o.off(blk, kSubwaveMaxClass + 1) - o.off(blk, 4);      // rows of 8 and more entries
        if (n_longer * 1000 >= n_sub) blocks = std::min<int64_t>(blocks, (int64_t)ctx->n_cu * PLX_SUB_PERSIST);
#endif
        k_spmm_subwave<T, G, VW><<<dim3((unsigned)blocks), 256, 0, s>>>(o.row_order + s0, n_sub, o.bptr + s0, o.col, o.val, X,
                                                                         ldx, out, d);
    }
    if (n_wave > 0) {
        KernelTimer kt(ctx, timed ? std::string("spmm_wave") + label : std::string(), timed);
        int64_t blocks = ceil_div(n_wave, WPB);
        k_spmm_wave<T, G, VW><<<dim3((unsigned)blocks), 256, 0, s>>>(o.row_order + s0 + n_sub, n_wave, o.bptr + s0 + n_sub, o.col,
                                                                      o.val, X, ldx, out, d);
    }
    PLX_HIP(ctx, hipGetLastError());
    return PLX_OK;
}

// Rows cut into segments: partial sums per segment, then the sums of each row in segment order.
template <typename T, int G, int VW>
plx_status run_long(plx_ctx* ctx, const Orient& o, int blk, const T* X, int64_t ldx, Out<T> out, int d, float* part, bool timed) {
    hipStream_t s = ctx->stream;
    const int64_t n_long = o.long0[blk + 1] - o.long0[blk], l0 = o.long0[blk];
    const int64_t n_seg = o.seg0b[blk + 1] - o.seg0b[blk], g0 = o.seg0b[blk];
    if (n_seg <= 0) return PLX_OK;
    char label[64];
    if (timed) snprintf(label, sizeof label, "<%s,G%d,VW%d,d%d>[%s]", sizeof(T) == 4 ? "f32" : "bf16", G, VW, d, o.tag ? "At" : "A");
    KernelTimer kt(ctx, timed ? std::string("spmm_split") + label : std::string(), timed);
    k_spmm_segment<T, G, VW><<<dim3((unsigned)ceil_div(n_seg, WPB)), 256, 0, s>>>(n_seg, o.seg_desc + g0, o.col, o.val, X, ldx, part, d);
    const int64_t total = n_long * d;
    k_spmm_combine<T><<<dim3((unsigned)ceil_div(total, 256)), 256, 0, s>>>(n_long, o.long_row + l0, o.long_seg0 + l0, part,
                                                                           G * VW, out, d);
    PLX_HIP(ctx, hipGetLastError());
    return PLX_OK;
}

template <typename T, int VW, bool LONG>
plx_status dispatch(plx_ctx* ctx, const Orient& o, int blk, const T* X, int64_t ldx, Out<T> out, int d, float* part, bool timed) {
    int G = 1;
    while (G * VW < d) G <<= 1;
#define PLX_SPMM_CASE(GV)                                                                    \
    case GV:                                                                                 \
        if constexpr (LONG) return run_long<T, GV, VW>(ctx, o, blk, X, ldx, out, d, part, timed); \
        else return run_short<T, GV, VW>(ctx, o, blk, X, ldx, out, d, timed)
    switch (G) {
        PLX_SPMM_CASE(1); PLX_SPMM_CASE(2); PLX_SPMM_CASE(4); PLX_SPMM_CASE(8); PLX_SPMM_CASE(16); PLX_SPMM_CASE(32);
        default: if constexpr (LONG) return run_long<T, 64, VW>(ctx, o, blk, X, ldx, out, d, part, timed);
                 else return run_short<T, 64, VW>(ctx, o, blk, X, ldx, out, d, timed);
    }
#undef PLX_SPMM_CASE
}

template <typename T, int VW>
plx_status run_vw(plx_ctx* ctx, const Orient& o, int block, const T* X, int64_t ldx, Out<T> out, int64_t d, const Partials& pt) {
    const bool timed = ctx->timing && !pt.given;
    const int tile = kWave * VW;                        // widest pass one wavefront covers
    // the segment kernels work in passes of at most this many columns: what a segment's slot of partial sums holds
    int64_t part_floats = kPartFloats;
    float* part = o.part;
    if (pt.given) {         // the same pass widths as with the handle's buffer (the results are then bit-identical), if they fit
        part = pt.given;
        if (o.n_seg > 0) part_floats = std::min<int64_t>(part_floats, (int64_t)(pt.bytes / sizeof(float)) / o.n_seg);
    }
    int long_tile = VW;
    while (2 * long_tile <= std::min<int64_t>(part_floats, tile)) long_tile *= 2;
    const int b_lo = block < 0 ? 0 : block, b_hi = block < 0 ? o.n_blocks : block + 1;
    for (int blk = b_lo; blk < b_hi; ++blk) {
        for (int64_t t0 = 0; t0 < d; t0 += tile) {
            const int dp = (int)std::min<int64_t>(tile, d - t0);
            Out<T> op{out.y ? out.y + t0 : nullptr, out.ldy, out.ya ? out.ya + t0 : nullptr, out.ldya};
            PLX_TRY((dispatch<T, VW, false>(ctx, o, blk, X + t0, ldx, op, dp, nullptr, timed)));
        }
        if (o.seg0b[blk + 1] - o.seg0b[blk] <= 0) continue;
        for (int64_t t0 = 0; t0 < d; t0 += long_tile) {
            const int dp = (int)std::min<int64_t>(long_tile, d - t0);
            Out<T> op{out.y ? out.y + t0 : nullptr, out.ldy, out.ya ? out.ya + t0 : nullptr, out.ldya};
            PLX_TRY((dispatch<T, VW, true>(ctx, o, blk, X + t0, ldx, op, dp, part, timed)));
        }
    }
    return PLX_OK;
}

bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Fixed buffer for the partial sums of split rows, for callers that cannot allocate (plx_spmm_static).  Every GPU
// the library runs on holds its own copy of this array, at its own address, until the process ends.  In host code
// the array's name is only a stand-in for hipGetSymbolAddress: kernels are given the resolved address.
constexpr size_t kStaticPartialsBytes = size_t(32) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticPartialsBytes];

constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
float* g_static_ptr[kMaxDevices];       // per device ordinal, resolved with that device current

}  // namespace

bool spmm_combine_supported(const Orient& o, const void* X, int64_t ldx, const void* S, int64_t lds_, int64_t din, int64_t dout,
                            plx_dtype dtype) {
    return dtype == PLX_F32 && din > 16 && din <= 32 && dout > 0 && dout <= 128 && o.n_blocks == 1 && o.long_class == kSubwaveMaxClass + 1 &&
           aligned_to(X, 16) && ldx % 4 == 0 && aligned_to(S, 16) && lds_ % 4 == 0;
}

plx_status launch_spmm_combine(plx_ctx* ctx, const Orient& o, const void* X, int64_t ldx, void* S, int64_t lds_, const float* W,
                               int64_t ldw, int64_t din, int64_t dout, void* C, int64_t ldc, void* Fact, int64_t ldf, uint32_t* bits,
                               int64_t ldbits) {
    if (!spmm_combine_supported(o, X, ldx, S, lds_, din, dout, PLX_F32)) return fail(ctx, PLX_ERR_INTERNAL, "fused aggregation outside its range");
    hipStream_t s = ctx->stream;
    const float* x = static_cast<const float*>(X);
    float* sp = static_cast<float*>(S);
    float* c = static_cast<float*>(C);
    float* f = static_cast<float*>(Fact);
    const int tnb = (int)ceil_div(dout, 32);
    const int64_t n_sub = o.off(0, kSubwaveMaxClass + 1) - o.off(0, 0);
    char label[96];
    snprintf(label, sizeof label, "<f32,d%lld,N%lld>[%s]", (long long)din, (long long)dout, o.tag ? "At" : "A");
    auto launch = [&](auto tag) -> plx_status {
        constexpr int TNB = decltype(tag)::value;
        const size_t lds = EpiLds<TNB>::bytes;
        if (n_sub > 0) {
            KernelTimer kt(ctx, ctx->timing ? std::string("spmm_subwave_combine") + label : std::string());
            const int64_t blocks = std::min<int64_t>(ceil_div(ceil_div(n_sub, 8), WPB), (int64_t)ctx->n_cu * PLX_SUB_PERSIST);
            k_spmm_subwave_combine<TNB><<<dim3((unsigned)blocks), 256, lds, s>>>(o.row_order, n_sub, o.bptr, o.col, o.val, x, ldx, sp, lds_,
                                                                                W, ldw, (int)din, (int)dout, c, ldc, f, ldf, bits, ldbits);
        }
        if (o.n_long > 0) {
            Out<float> out{sp, lds_, nullptr, 0};
            PLX_TRY((dispatch<float, 4, true>(ctx, o, 0, x, ldx, out, (int)din, o.part, ctx->timing)));   // segments, then the rows' sums
            KernelTimer kt(ctx, ctx->timing ? std::string("rows_combine") + label : std::string());
            k_rows_combine<TNB><<<dim3((unsigned)ceil_div(ceil_div(o.n_long, kEpiRows), WPB)), 256, lds, s>>>(
                o.n_long, o.long_row, sp, lds_, W, ldw, (int)din, (int)dout, c, ldc, f, ldf, bits, ldbits);
        }
        PLX_HIP(ctx, hipGetLastError());
        return PLX_OK;
    };
    switch (tnb) {
        case 1: return launch(std::integral_constant<int, 1>{});
        case 2: return launch(std::integral_constant<int, 2>{});
        case 3: return launch(std::integral_constant<int, 3>{});
        default: return launch(std::integral_constant<int, 4>{});
    }
}

float* static_partials(plx_ctx* ctx, size_t* bytes) {
    if (bytes) *bytes = kStaticPartialsBytes;
    if (ctx->dry || ctx->device < 0 || ctx->device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[ctx->device]) {
        int current = -1;
        if (hipGetDevice(&current) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
        if (current != ctx->device && hipSetDevice(ctx->device) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (current != ctx->device) (void)hipSetDevice(current);
        if (e != hipSuccess || !p) { (void)hipGetLastError(); return nullptr; }
        g_static_ptr[ctx->device] = static_cast<float*>(p);
    }
    return g_static_ptr[ctx->device];
}

plx_status launch_spmm(plx_ctx* ctx, const Orient& o, const void* X, int64_t ldx, void* Y, int64_t ldy, int64_t d,
                       plx_dtype dtype, void* Yact, int64_t ldyact, int block, float* partials, size_t partials_bytes) {
    Partials pt;
    pt.given = partials; pt.bytes = partials_bytes;
    if (o.rows >= (int64_t(1) << 31) || o.nnz >= (int64_t(1) << 31))
        return fail(ctx, PLX_ERR_UNSUPPORTED, "matrix too large for 32-bit ids");
    // widest vector the layout allows: base pointers and row pitches must keep every row aligned
    auto fits = [&](size_t bytes, size_t es) {
        return aligned_to(X, bytes) && (ldx * es) % bytes == 0 &&
               (!Y || (aligned_to(Y, bytes) && (ldy * es) % bytes == 0)) &&
               (!Yact || (aligned_to(Yact, bytes) && (ldyact * es) % bytes == 0));
    };
    if (o.n_seg > 0) {
        // checked before anything is queued: a segment's partial sums need room for at least one vector per lane group
        const int vw = dtype == PLX_F32 ? (fits(16, 4) ? 4 : fits(8, 4) ? 2 : 1) : (fits(16, 2) ? 8 : fits(8, 2) ? 4 : 1);
        if (partials) {
            const int64_t dp = std::min<int64_t>(d, std::min<int64_t>((int64_t)kWave * vw, kPartFloats));
            int64_t g = 1;
            while (g * vw < dp) g <<= 1;
            const size_t need = (size_t)o.n_seg * (size_t)(g * vw) * sizeof(float);
            if (need > partials_bytes)
                return fail(ctx, PLX_ERR_UNSUPPORTED, "the partial sums of %lld segments at width %lld take %zu bytes, more than the "
                            "%zu bytes of the fixed buffer", (long long)o.n_seg, (long long)d, need, partials_bytes);
        } else if (!o.part) {
            return fail(ctx, PLX_ERR_INTERNAL, "the handle holds segments but no buffer for their partial sums");
        }
    }
    if (dtype == PLX_F32) {
        const float* x = static_cast<const float*>(X);
        Out<float> out{static_cast<float*>(Y), ldy, static_cast<float*>(Yact), ldyact};
        if (fits(16, 4)) return run_vw<float, 4>(ctx, o, block, x, ldx, out, d, pt);
        if (fits(8, 4)) return run_vw<float, 2>(ctx, o, block, x, ldx, out, d, pt);
        return run_vw<float, 1>(ctx, o, block, x, ldx, out, d, pt);
    }
    const bf16_t* x = static_cast<const bf16_t*>(X);
    Out<bf16_t> out{static_cast<bf16_t*>(Y), ldy, static_cast<bf16_t*>(Yact), ldyact};
    if (fits(16, 2)) return run_vw<bf16_t, 8>(ctx, o, block, x, ldx, out, d, pt);
    if (fits(8, 2)) return run_vw<bf16_t, 4>(ctx, o, block, x, ldx, out, d, pt);
    return run_vw<bf16_t, 1>(ctx, o, block, x, ldx, out, d, pt);
}

}  // namespace plx
