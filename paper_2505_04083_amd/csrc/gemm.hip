// Dense products of a GCN layer on the matrix cores (paper Eq. 2.2 Q = H W, Eq. 2.6
// dH = dQ W^T, Eq. 2.5 dW = H^T dQ).  One operand is always tall and skinny (N_nodes x <=602),
// the other a small weight matrix, so these products stream the tall operand once from HBM
// and are bound by that stream; MFMA does the arithmetic so the vector ALUs stay free.
//
// fp32 path: v_mfma_f32_32x32x2_f32.  Operand layout of that instruction for lane l:
//   a = A[i = l % 32][k = l / 32],  b = B[k = l / 32][j = l % 32],
//   acc[r] = C[i = 8*(r/4) + 4*(l/32) + r%4][j = l % 32],  r = 0..15.
// General kernels (any K, N): a workgroup of 4 wavefronts owns a tile of TMB x TNB such 32x32
// blocks; block q of the tile (row-major) belongs to wavefront q % 4; slabs of 32 values of k of
// both operands are staged through LDS.  Operands with 16-byte aligned rows take the variant with
// buffer loads, two LDS buffers and one barrier per slab (measured on 232965 x 602 by 602 x 128:
// 68 % of the fp32 matrix peak against 37 % for the element-wise guarded one, which stays for
// unaligned rows).  Layer-sized products (K, N <= 128) take the persistent kernel further down,
// which keeps the weights in registers.
//
// Where K and N both exceed 32 the persistent kernel forms its fp32 products from six bf16 matrix
// products each (k_gemm_small_x3); that kernel can also multiply its result tile by the weights
// of a following combine-first layer on the way out (T = F Wn), so that layer does not read F back.
//
// The transposed product (reduction over the node dimension) is split over row chunks; each
// workgroup writes its partial tile and a second kernel adds the partials in a fixed order, so
// the result does not depend on scheduling.
#include "plx_internal.h"
#include "buffer_addr.h"
#include "bf16_frag.h"

#include <algorithm>
#include <type_traits>

namespace plx {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kBK = 32;   // depth of one staged slab

__device__ __forceinline__ floatx16 mfma32(float a, float b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// ---- C[M x N] = A[M x K] * B  (B is K x N, or N x K when BT) -------------------------------------
template <int TNB, bool BT>
__global__ __launch_bounds__(256) void k_gemm_f32(int64_t M, int N, int K, const float* __restrict__ A, int64_t lda,
                                                  const float* __restrict__ B, int64_t ldb, float* __restrict__ C,
                                                  int64_t ldc, float* __restrict__ F, int64_t ldf, int vec_a) {
    constexpr int TMB = 4;
    constexpr int BM = 32 * TMB, BN = 32 * TNB;
    constexpr int NBLK = TMB * TNB / 4;               // blocks per wavefront
    __shared__ float As[BM][kBK + 1];
    __shared__ float Bs[kBK][BN + 1];
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;

    floatx16 acc[NBLK];
#pragma unroll
    for (int t = 0; t < NBLK; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

    // Slabs of kBK columns of A and rows of B go global -> registers -> LDS; the loads of the next
    // slab are in flight while the matrix cores work on the current one (the last pass re-reads
    // its own slab, so the loop body has no condition around the prefetch).
    constexpr int NA = (BM * kBK / 4) / 256, NB = (kBK * BN) / 256;
    float4 ra[NA];
    float rb[NB];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int f = tid + 256 * i, r = f >> 3, q = f & 7;
            const int64_t gr = m0 + r;
            const int gk = k0 + 4 * q;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (gr < M) {
                const float* p = A + gr * lda + gk;
                if (vec_a && gk + 3 < K) {
                    v = *reinterpret_cast<const float4*>(p);
                } else {
                    if (gk < K) v.x = p[0];
                    if (gk + 1 < K) v.y = p[1];
                    if (gk + 2 < K) v.z = p[2];
                    if (gk + 3 < K) v.w = p[3];
                }
            }
            ra[i] = v;
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int f = tid + 256 * i;
            int kk, n;
            if (BT) { n = f / kBK; kk = f % kBK; } else { kk = f / BN; n = f % BN; }
            const int gk = k0 + kk, gn = n0 + n;
            float v = 0.f;
            if (gk < K && gn < N) v = BT ? B[(int64_t)gn * ldb + gk] : B[(int64_t)gk * ldb + gn];
            rb[i] = v;
        }
    };
    auto commit = [&]() {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int f = tid + 256 * i, r = f >> 3, q = f & 7;
            As[r][4 * q + 0] = ra[i].x; As[r][4 * q + 1] = ra[i].y; As[r][4 * q + 2] = ra[i].z; As[r][4 * q + 3] = ra[i].w;
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int f = tid + 256 * i;
            int kk, n;
            if (BT) { n = f / kBK; kk = f % kBK; } else { kk = f / BN; n = f % BN; }
            Bs[kk][n] = rb[i];
        }
    };
    fetch(0);
    commit();
    __syncthreads();
    for (int k0 = 0; k0 < K; k0 += kBK) {
        fetch(k0 + kBK < K ? k0 + kBK : k0);
#pragma unroll 4
        for (int kk = 0; kk < kBK; kk += 2) {
#pragma unroll
            for (int t = 0; t < NBLK; ++t) {       // TMB * TNB is a multiple of 4: every block index is valid
                const int q = w + 4 * t, bi = q / TNB, bj = q % TNB;
                acc[t] = mfma32(As[32 * bi + l32][kk + lh], Bs[kk + lh][32 * bj + l32], acc[t]);
            }
        }
        __syncthreads();                           // every wavefront is done with the slab
        commit();
        __syncthreads();
    }
#pragma unroll
    for (int t = 0; t < NBLK; ++t) {
        const int q = w + 4 * t, bi = q / TNB, bj = q % TNB;
        const int gn = n0 + 32 * bj + l32;
        if (gn >= N) continue;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t gr = m0 + 32 * bi + 8 * (r / 4) + 4 * lh + (r % 4);
            if (gr < M) {
                const float v = acc[t][r];
                if (C) C[gr * ldc + gn] = v;
                if (F) F[gr * ldf + gn] = v > 0.f ? v : 0.f;      // Eq. 2.3 fused into the store
            }
        }
    }
}

// ---- the same product for 16-byte aligned operands: buffer loads, two LDS buffers, one barrier per slab ----
// Tile 128 x 32*TNB; wavefront w owns the column block w % TNB of TNB row blocks.  A slab is 32 values
// of k; the next one travels global -> registers while the matrix cores work on the current one and
// is written to the other LDS buffer afterwards, so a slab costs one barrier.  The A tile (and the
// B tile when BT, whose rows are then k-contiguous as well) is read from LDS 128 bits at a time:
// instruction j of a group of four takes k = 8g + 4*(l/32) + j (any order of k gives the same sum).
// Every address step inside the loop is scalar: the lane offsets are computed once.
// TA = bf16_t: A, C and F hold bf16; A is widened on its way into LDS (exact), so the products are
// those of the fp32 kernel on bf16-valued inputs, and the results are rounded to nearest even.

// a 16-byte piece of a row as fp32 values: 4 of an fp32 row, 8 of a bf16 row
template <typename T> struct RowPiece;
template <> struct RowPiece<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void widen(const float4& raw, float4 (&v)[1]) { v[0] = raw; }
};
template <> struct RowPiece<bf16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void widen(const float4& raw, float4 (&v)[2]) {
        const uint4 u = __builtin_bit_cast(uint4, raw);
        v[0] = make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u), __uint_as_float(u.y << 16),
                           __uint_as_float(u.y & 0xffff0000u));
        v[1] = make_float4(__uint_as_float(u.z << 16), __uint_as_float(u.z & 0xffff0000u), __uint_as_float(u.w << 16),
                           __uint_as_float(u.w & 0xffff0000u));
    }
};
// A piece whose values straddle the end of the reduction keeps only those before it: what lies behind
// them in memory (padding, the next row) need not be finite, and 0 * NaN would reach a whole output row.
__device__ __forceinline__ void clip_piece(float4& v, int left) {
    v.x = left > 0 ? v.x : 0.f; v.y = left > 1 ? v.y : 0.f; v.z = left > 2 ? v.z : 0.f; v.w = left > 3 ? v.w : 0.f;
}
// bytes up to and including element (last_row, cols - 1) of a matrix of T, rounded up to the 4-byte
// granularity of the range check (bf16 rows are padded to 16 bytes, so the extra element exists)
template <typename T>
__device__ __forceinline__ uint32_t extent_bytes(int last_row, int64_t ld, int cols) {
    return (uint32_t)((((int64_t)last_row * ld + cols) * (int64_t)sizeof(T) + 3) & ~int64_t(3));
}
__device__ __forceinline__ void store_elt(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t row_off, float v, float*) {
    buffer_store(r, lane_off, row_off, v);
}
__device__ __forceinline__ void store_elt(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t row_off, float v, bf16_t*) {
    __builtin_amdgcn_raw_buffer_store_b16((short)f32_to_bf16(v), r, (int)lane_off, (int)row_off, 0);
}

template <int TNB, bool BT, typename TA, bool BV>   // BV: the rows of B are 16-byte aligned as well (else four 4-byte loads per piece)
__global__ __launch_bounds__(256) void k_gemm_deep(int64_t M, int N, int K, const TA* __restrict__ A, int64_t lda,
                                                   const float* __restrict__ B, int64_t ldb, TA* __restrict__ C,
                                                   int64_t ldc, TA* __restrict__ F, int64_t ldf) {
    constexpr int BM = 128, BN = 32 * TNB, AP = kBK + 4;
    constexpr int BROWS = BT ? BN : kBK, BP = BT ? kBK + 4 : BN + 4;   // the B tile as it lies in memory
    constexpr int NE = RowPiece<TA>::N, PPR = kBK / NE;                // elements per piece, pieces per row of an A slab
    constexpr int NA = BM * PPR / 256, NBV = BN * kBK / 4 / 256;       // 16-byte pieces per thread and slab
    constexpr int NBLK = TNB;                                          // 4 * TNB blocks over 4 wavefronts
    constexpr uint32_t ES = sizeof(TA);
    extern __shared__ __align__(16) float smem[];
    typedef float (*ATile)[AP];
    typedef float (*BTile)[BP];
    auto a_buf = [&](int b) { return reinterpret_cast<ATile>(smem + b * BM * AP); };
    auto b_buf = [&](int b) { return reinterpret_cast<BTile>(smem + 2 * BM * AP + b * BROWS * BP); };
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;
    const int rows = (int)(M - m0 < BM ? M - m0 : BM), cols = N - n0 < BN ? N - n0 : BN;
    const int bj = w % TNB;
    auto row_block = [&](int t) { return (w + 4 * t) / TNB; };

    uint32_t offa[NA], offb[NBV];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int f = tid + 256 * i, r = f / PPR, q = f % PPR;
        offa[i] = ((uint32_t)r * (uint32_t)lda + (uint32_t)(NE * q)) * ES;
    }
#pragma unroll
    for (int i = 0; i < NBV; ++i) {
        const int f = tid + 256 * i;
        const int r = BT ? f >> 3 : f / (BN / 4), q = BT ? f & 7 : f % (BN / 4);
        offb[i] = (uint32_t)(((uint32_t)r * (uint32_t)ldb + 4u * q) * 4u);
    }
    const int ka = NE * (tid % PPR), kb = 4 * (tid & 7);     // first k of a thread's pieces inside a slab (B: when BT)
    const TA* a_row = A + m0 * lda;
    const float* b_base = BT ? B + (int64_t)n0 * ldb : B + n0;

    float4 ra[NA], rb[NBV];
    int kleft_fetched = 0;                                   // K - k0 of the slab the registers hold
    auto load_b = [&](__amdgpu_buffer_rsrc_t d, uint32_t off) {
        if constexpr (BV) return buffer_load4(d, off);
        else   // the range check is per 4-byte word, so the four words of a piece may end anywhere in a row
            return make_float4(__uint_as_float(buffer_load1(d, off)), __uint_as_float(buffer_load1(d, off + 4)),
                               __uint_as_float(buffer_load1(d, off + 8)), __uint_as_float(buffer_load1(d, off + 12)));
    };
    auto fetch = [&](int k0) {
        const int kleft = K - k0;                            // > 0
        kleft_fetched = kleft;
        // byte counts end with the last valid element: rows past the end of a matrix read as 0
        const __amdgpu_buffer_rsrc_t da = buffer_of(a_row + k0, extent_bytes<TA>(rows - 1, lda, kleft));
#pragma unroll
        for (int i = 0; i < NA; ++i) ra[i] = buffer_load4(da, offa[i]);
        if constexpr (BT) {
            const __amdgpu_buffer_rsrc_t db = buffer_of(b_base + k0, extent_bytes<float>(cols - 1, ldb, kleft));
#pragma unroll
            for (int i = 0; i < NBV; ++i) rb[i] = load_b(db, offb[i]);
        } else {
            const int krows = kleft < kBK ? kleft : kBK;
            const __amdgpu_buffer_rsrc_t db = buffer_of(b_base + (int64_t)k0 * ldb, extent_bytes<float>(krows - 1, ldb, cols));
#pragma unroll
            for (int i = 0; i < NBV; ++i) rb[i] = load_b(db, offb[i]);
        }
    };
    auto commit = [&](int b) {
        ATile As = a_buf(b);
        BTile Bs = b_buf(b);
        const bool tail = kleft_fetched < kBK;               // uniform: the last slab of a K that is no multiple of 32
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int f = tid + 256 * i;
            float4 v[NE / 4];
            RowPiece<TA>::widen(ra[i], v);
#pragma unroll
            for (int j = 0; j < NE / 4; ++j) {
                if (tail) clip_piece(v[j], kleft_fetched - ka - 4 * j);
                *reinterpret_cast<float4*>(&As[f / PPR][NE * (f % PPR) + 4 * j]) = v[j];
            }
        }
#pragma unroll
        for (int i = 0; i < NBV; ++i) {
            const int f = tid + 256 * i;
            const int r = BT ? f >> 3 : f / (BN / 4), q = BT ? f & 7 : f % (BN / 4);
            if (BT && tail) clip_piece(rb[i], kleft_fetched - kb);
            *reinterpret_cast<float4*>(&Bs[r][4 * q]) = rb[i];
        }
    };

    floatx16 acc[NBLK];
#pragma unroll
    for (int t = 0; t < NBLK; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

    fetch(0);
    commit(0);
    __syncthreads();
    int cur = 0;
    for (int k0 = 0; k0 < K; k0 += kBK) {
        fetch(k0 + kBK < K ? k0 + kBK : k0);       // no condition around the prefetch: the last pass re-reads its own slab
        ATile As = a_buf(cur);
        BTile Bs = b_buf(cur);
#pragma unroll
        for (int g = 0; g < kBK / 8; ++g) {
            float4 b4;
            if constexpr (BT) {
                b4 = *reinterpret_cast<const float4*>(&Bs[32 * bj + l32][8 * g + 4 * lh]);
            } else {
                b4.x = Bs[8 * g + 4 * lh + 0][32 * bj + l32];
                b4.y = Bs[8 * g + 4 * lh + 1][32 * bj + l32];
                b4.z = Bs[8 * g + 4 * lh + 2][32 * bj + l32];
                b4.w = Bs[8 * g + 4 * lh + 3][32 * bj + l32];
            }
            float4 a4[NBLK];
#pragma unroll
            for (int t = 0; t < NBLK; ++t) a4[t] = *reinterpret_cast<const float4*>(&As[32 * row_block(t) + l32][8 * g + 4 * lh]);
#pragma unroll
            for (int t = 0; t < NBLK; ++t) {
                acc[t] = mfma32(a4[t].x, b4.x, acc[t]);
                acc[t] = mfma32(a4[t].y, b4.y, acc[t]);
                acc[t] = mfma32(a4[t].z, b4.z, acc[t]);
                acc[t] = mfma32(a4[t].w, b4.w, acc[t]);
            }
        }
        commit(cur ^ 1);                           // the barrier of the pass before ended every read of that buffer
        __syncthreads();
        cur ^= 1;
    }

    const int gn = 32 * bj + l32;
    if (gn < cols) {
        // lane part of an address: column, and the +4 rows of the upper half-wave; the row part is scalar
        const uint32_t coff = (4u * lh * (uint32_t)ldc + gn) * ES, foff = (4u * lh * (uint32_t)ldf + gn) * ES;
        const __amdgpu_buffer_rsrc_t rc = buffer_of(C ? C + m0 * ldc + n0 : nullptr, extent_bytes<TA>(BM - 1, ldc, cols));
        const __amdgpu_buffer_rsrc_t rf = buffer_of(F ? F + m0 * ldf + n0 : nullptr, extent_bytes<TA>(BM - 1, ldf, cols));
        auto emit = [&](auto guarded, auto has_c, auto has_f) {
#pragma unroll
            for (int t = 0; t < NBLK; ++t) {
                const int rb0 = 32 * row_block(t);                                   // scalar
                uint32_t crow = (uint32_t)rb0 * (uint32_t)ldc * ES, frow = (uint32_t)rb0 * (uint32_t)ldf * ES;
                int at = 0;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = 8 * (r / 4) + (r % 4);                           // of the lower half-wave, inside the block
                    crow += (uint32_t)(row - at) * (uint32_t)ldc * ES;
                    frow += (uint32_t)(row - at) * (uint32_t)ldf * ES;
                    at = row;
                    const float v = acc[t][r];
                    if (!guarded.value || rb0 + row + 4 * lh < rows) {
                        if (has_c.value) store_elt(rc, coff, crow, v, C);
                        if (has_f.value) store_elt(rf, foff, frow, relu0(v), F);     // Eq. 2.3 fused into the store
                    }
                }
            }
        };
        auto emit_cf = [&](auto guarded) {
            if (C && F) emit(guarded, std::true_type{}, std::true_type{});
            else if (F) emit(guarded, std::false_type{}, std::true_type{});
            else emit(guarded, std::true_type{}, std::false_type{});
        };
        if (rows == BM) emit_cf(std::false_type{}); else emit_cf(std::true_type{});
    }
}

// ---- C[M x N] = A[M x K] * B[K x N] for K, N <= 128: persistent row loop, weights in registers ------
// A workgroup walks over TR-row tiles of A (tile index strided by the grid).  Every wavefront keeps
// its share of the weight matrix in registers, already in the lane layout the matrix instruction
// wants, for the whole kernel; LDS holds only the double-buffered tile of A, so several workgroups
// fit on a CU and their load, MFMA and store phases overlap.  The next tile is fetched into
// registers while the matrix cores work on the current one.  Output: C and / or max(C, 0).
//
// N > 64 (WIDE): v_mfma_f32_32x32x2_f32; wavefront w owns the 32-column block w (N padded to 128)
//   of every 32-row block of the tile; lane l holds b[s] = B[k(s, l/32)][32w + l%32] with the k order
//   chosen so that four consecutive instructions read one 128-bit piece of an A row from LDS.
// N <= 64: v_mfma_f32_16x16x4_f32 (N padded to 16 only); lane l supplies a = A[row l%16][4s + l/16],
//   b = B[4s + l/16][16c + l%16] and receives acc[r] = C[4*(l/16) + r][16c + l%16].  With 64-row
//   tiles wavefront w owns row block w and every column block; with 32-row tiles (taken when the
//   weight registers would not fit otherwise) row block w%2 and column blocks w/2 and w/2 + 2.
typedef float floatx4 __attribute__((ext_vector_type(4)));

// Results are written once and read by a later kernel after gigabytes of other traffic: they leave
// through non-temporal buffer stores, which keeps them from displacing cache lines that are still
// useful (measured: -6 %).
#ifndef PLX_FWD_WIDE_TR_K128
#define PLX_FWD_WIDE_TR_K128 32
#endif
#ifndef PLX_FWD_WIDE_TR
#define PLX_FWD_WIDE_TR 64
#endif
// rows per tile for a (K, N) class: 32 when 64 would need too many registers for the weights
constexpr int fwd_tile_rows(int tkb, int cb) {
    if (cb > 4) return tkb == 4 ? PLX_FWD_WIDE_TR_K128 : PLX_FWD_WIDE_TR;
    return cb * (32 * tkb / 4) > 64 ? 32 : 64;
}

template <int TKB, int CB, bool VEC>   // K <= 32*TKB; N <= 16*CB (CB <= 4) or N <= 128 (CB == 8); VEC: 16-byte aligned rows, K % 4 == 0
__global__ __launch_bounds__(256) void k_gemm_small_f32(int64_t M, int N, int K, const float* __restrict__ A,
                                                        int64_t lda, const float* __restrict__ B, int64_t ldb,
                                                        float* __restrict__ C, int64_t ldc, float* __restrict__ F,
                                                        int64_t ldf, uint32_t* __restrict__ bits, int64_t ldbits,
                                                        int bits_vec) {
    constexpr bool WIDE = CB > 4;
    constexpr int TR = fwd_tile_rows(TKB, CB);
    constexpr int KP = 32 * TKB;
    constexpr int NLD = TR * KP / 4 / 256;                               // float4 per thread per tile
    constexpr int NRB = WIDE ? TR / 32 : 1;                              // row blocks per wavefront
    constexpr int NCW = WIDE ? 1 : (TR == 64 ? CB : (CB + 1) / 2);       // column blocks per wavefront
    constexpr int KSTEP = WIDE ? 2 : 4, NKS = KP / KSTEP, CHUNK = 8;     // k per instruction, instructions, guard granularity
    static_assert(NLD >= 1 && NKS % CHUNK == 0, "tile shape");
    extern __shared__ __align__(16) float smem[];
    // two A buffers: the next tile is written to LDS before this tile's stores are issued
    typedef float (*ATile)[KP + 4];
    auto a_buf = [&](int b) { return reinterpret_cast<ATile>(smem + b * TR * (KP + 4)); };
    // Sign bits of a tile (only when bits != NULL): the wavefronts drop their ballots into LDS and the
    // words leave one tile later as one store per row.  Two buffers of TR rows x 4 words; WIDE keeps
    // them word-major ([word][row]: a lane's four consecutive rows are one 128-bit LDS write), the
    // narrow tiles row-major as 8 half-words per row (a 16-column block is one half-word).
    uint32_t* sb = reinterpret_cast<uint32_t*>(smem + 2 * TR * (KP + 4));
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lq = lane >> 4, l32 = lane & 31, lh = lane >> 5;
    const int k_end = (K + KSTEP - 1) / KSTEP * KSTEP;
    const int rowblk = WIDE ? 0 : (TR == 64 ? w : (w & 1));
    auto col_block = [&](int c) { return WIDE ? w : (TR == 64 ? c : (w >> 1) + 2 * c); };

    float breg[NCW][NKS];
#pragma unroll
    for (int c = 0; c < NCW; ++c) {
        const int n = WIDE ? 32 * w + l32 : 16 * col_block(c) + l16;
#pragma unroll
        for (int s = 0; s < NKS; ++s) {
            // WIDE: instruction s of a group of four takes k = 8*(s/4) + 4*(l/32) + s%4, so that a lane's
            // four A values of the group are one 128-bit LDS read (any order of k gives the same sum)
            const int kk = WIDE ? 8 * (s / 4) + 4 * lh + (s % 4) : 4 * s + lq;
            breg[c][s] = (kk < K && n < N) ? B[(int64_t)kk * ldb + n] : 0.f;
        }
    }
    // The weights must have landed before the row loop starts: otherwise their first use inside the
    // loop waits for ALL outstanding loads, the freshly issued prefetch of the next tile included.
    __builtin_amdgcn_s_waitcnt(0x0F70);    // vmcnt(0), other counters untouched

    const int64_t n_tiles = (M + TR - 1) / TR;
    float4 reg[NLD];
    uint32_t toff[NLD];                    // VEC: byte offset of a thread's 16-byte pieces inside a tile
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int f = tid + 256 * i, r = f / (KP / 4), q = f % (KP / 4);
        toff[i] = (KP == K || 4 * q < K) ? (uint32_t)(((uint32_t)r * (uint32_t)lda + 4u * q) * 4u) : kOutOfRange;
    }
    const uint32_t tile_bytes_a = (uint32_t)(((TR - 1) * lda + K) * 4);
    auto fetch = [&](int64_t tile) {
        const int64_t m0 = tile * TR;
        if constexpr (VEC) {               // the byte count ends with the last valid row: rows past it read as 0
            const int64_t left = M - m0;
            const __amdgpu_buffer_rsrc_t ra = buffer_of(A + m0 * lda, left >= TR ? tile_bytes_a : (uint32_t)(((left - 1) * lda + K) * 4));
#pragma unroll
            for (int i = 0; i < NLD; ++i) reg[i] = buffer_load4(ra, toff[i]);
            return;
        }
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int f = tid + 256 * i, r = f / (KP / 4), q = f % (KP / 4);
            const int64_t gr = m0 + r;
            const int gk = 4 * q;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (gr < M && gk < K) {
                const float* p = A + gr * lda + gk;
                v.x = p[0];
                if (gk + 1 < K) v.y = p[1];
                if (gk + 2 < K) v.z = p[2];
                if (gk + 3 < K) v.w = p[3];
            }
            reg[i] = v;
        }
    };
    auto commit = [&](ATile As) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int f = tid + 256 * i, r = f / (KP / 4), q = f % (KP / 4);
            *reinterpret_cast<float4*>(&As[r][4 * q]) = reg[i];
        }
    };

    const int nw = (N + 31) >> 5;
    auto flush_bits = [&](int buf, int64_t t) {                          // words of tile t, written by the pass before
        const int64_t row = t * TR + tid;
        if (tid < TR && row < M) {
            uint32_t wds[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) wds[j] = WIDE ? sb[(buf * 4 + j) * TR + tid] : sb[(buf * TR + tid) * 4 + j];
            uint32_t* dst = bits + row * ldbits;
            if (bits_vec == 4) *reinterpret_cast<uint4*>(dst) = make_uint4(wds[0], wds[1], wds[2], wds[3]);
            else if (bits_vec == 2) *reinterpret_cast<uint2*>(dst) = make_uint2(wds[0], wds[1]);
            else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (j < nw) dst[j] = wds[j];
            }
        }
    };

    int64_t tile = blockIdx.x, prev = -1;
    int cur = 0;
    if (bits)
        for (int i = tid; i < 2 * TR * 4; i += 256) sb[i] = 0;          // half-words no wavefront owns stay 0
    if (tile < n_tiles) { fetch(tile); commit(a_buf(0)); }
    __syncthreads();
    for (; tile < n_tiles; tile += gridDim.x) {
        // No condition around the prefetch and its LDS write (the last pass re-reads its own tile):
        // with straight-line code the only wait for loads sits right before the LDS write, after the
        // matrix work, and nothing ever waits for the previous tile's stores to be acknowledged.
        const bool more = tile + gridDim.x < n_tiles;
        fetch(more ? tile + gridDim.x : tile);
        if (bits && prev >= 0) flush_bits(cur ^ 1, prev);
        prev = tile;
        ATile As = a_buf(cur);
        const bool full = (tile + 1) * TR <= M;                         // uniform: only the last tile is partial

        if constexpr (WIDE) {
            floatx16 acc[NRB];
#pragma unroll
            for (int t = 0; t < NRB; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
#pragma unroll
            for (int s0 = 0; s0 < NKS; s0 += CHUNK) {
                if (s0 > 0 && KSTEP * s0 >= k_end) break;                // uniform: no matrix work on k-padding beyond a chunk
#pragma unroll
                for (int g = s0 / 4; g < (s0 + CHUNK) / 4; ++g) {
                    float4 a4[NRB];
#pragma unroll
                    for (int t = 0; t < NRB; ++t) a4[t] = *reinterpret_cast<const float4*>(&As[32 * t + l32][8 * g + 4 * lh]);
#pragma unroll
                    for (int t = 0; t < NRB; ++t) {
                        acc[t] = mfma32(a4[t].x, breg[0][4 * g + 0], acc[t]);
                        acc[t] = mfma32(a4[t].y, breg[0][4 * g + 1], acc[t]);
                        acc[t] = mfma32(a4[t].z, breg[0][4 * g + 2], acc[t]);
                        acc[t] = mfma32(a4[t].w, breg[0][4 * g + 3], acc[t]);
                    }
                }
            }
            commit(a_buf(cur ^ 1));
            const int gn = 32 * w + l32;
            if (gn < N) {
                // lane part of an address: column, and the +4 rows of the upper half-wave; the row part is scalar
                const uint32_t coff = (uint32_t)((4u * lh * (uint32_t)ldc + gn) * 4u), foff = (uint32_t)((4u * lh * (uint32_t)ldf + gn) * 4u);
                const int64_t m0 = tile * TR;
                const __amdgpu_buffer_rsrc_t rc = buffer_of(C ? C + m0 * ldc : nullptr, (uint32_t)(((TR - 1) * ldc + N) * 4));
                const __amdgpu_buffer_rsrc_t rf = buffer_of(F ? F + m0 * ldf : nullptr, (uint32_t)(((TR - 1) * ldf + N) * 4));
                auto emit = [&](auto guarded, auto has_c, auto has_f) {
                    uint32_t crow = opaque_zero(), frow = crow;                      // byte offset of the tile's row `row`
                    int at = 0;
#pragma unroll
                    for (int t = 0; t < NRB; ++t)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int row = 32 * t + 8 * (r / 4) + (r % 4);            // of the lower half-wave
                            crow += (uint32_t)(row - at) * (uint32_t)ldc * 4u;
                            frow += (uint32_t)(row - at) * (uint32_t)ldf * 4u;
                            at = row;
                            const float v = acc[t][r];
                            if (!guarded.value || m0 + row + 4 * lh < M) {
                                if (has_c.value) buffer_store_nt(rc, coff, crow, v);
                                if (has_f.value) buffer_store_nt(rf, foff, frow, relu0(v));   // Eq. 2.3 fused into the store
                            }
                        }
                };
                auto emit_cf = [&](auto guarded) {
                    if (C && F) emit(guarded, std::true_type{}, std::true_type{});
                    else if (F) emit(guarded, std::false_type{}, std::true_type{});
                    else emit(guarded, std::true_type{}, std::false_type{});
                };
                if (full) emit_cf(std::false_type{}); else emit_cf(std::true_type{});
            }
            if (bits) {       // one ballot = 32 columns of two rows (lanes 0-31: row dr, lanes 32-63: row dr + 4); columns >= N give 0
                // the ballots are wave-uniform (scalar registers): lane 0 alone stores both halves, 8 consecutive rows per step
                // (a per-lane choice between the halves turns into 64-bit vector shifts)
#pragma unroll
                for (int t = 0; t < NRB; ++t)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        uint32_t lo[4], hi[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const unsigned long long b = __ballot(acc[t][4 * g + j] > 0.f);
                            lo[j] = (uint32_t)b;
                            hi[j] = (uint32_t)(b >> 32);
                        }
                        if (lane == 0) {
                            uint4* dst = reinterpret_cast<uint4*>(&sb[(cur * 4 + w) * TR + 32 * t + 8 * g]);
                            dst[0] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
                            dst[1] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
                        }
                    }
            }
        } else {
            floatx4 acc[NCW];
#pragma unroll
            for (int c = 0; c < NCW; ++c) acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s0 = 0; s0 < NKS; s0 += CHUNK) {
                if (s0 > 0 && KSTEP * s0 >= k_end) break;
#pragma unroll
                for (int s = s0; s < s0 + CHUNK; ++s) {
                    const float a = As[16 * rowblk + l16][4 * s + lq];
#pragma unroll
                    for (int c = 0; c < NCW; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, breg[c][s], acc[c], 0, 0, 0);
                }
            }
            commit(a_buf(cur ^ 1));
            {
                const int64_t m0 = tile * TR;
                const __amdgpu_buffer_rsrc_t rc = buffer_of(C ? C + m0 * ldc : nullptr, (uint32_t)(((TR - 1) * ldc + N) * 4));
                const __amdgpu_buffer_rsrc_t rf = buffer_of(F ? F + m0 * ldf : nullptr, (uint32_t)(((TR - 1) * ldf + N) * 4));
                auto emit = [&](auto has_c, auto has_f) {
#pragma unroll
                    for (int c = 0; c < NCW; ++c) {
                        const int gn = 16 * col_block(c) + l16;
                        if (gn >= N) continue;
                        const uint32_t coff = (uint32_t)((4u * lq * (uint32_t)ldc + gn) * 4u), foff = (uint32_t)((4u * lq * (uint32_t)ldf + gn) * 4u);
                        uint32_t crow = opaque_zero() + 16u * rowblk * (uint32_t)ldc * 4u, frow = opaque_zero() + 16u * rowblk * (uint32_t)ldf * 4u;
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            if (full || m0 + 16 * rowblk + r + 4 * lq < M) {
                                const float v = acc[c][r];
                                if (has_c.value) buffer_store_nt(rc, coff, crow, v);
                                if (has_f.value) buffer_store_nt(rf, foff, frow, relu0(v));       // Eq. 2.3 fused into the store
                            }
                            crow += (uint32_t)ldc * 4u;
                            frow += (uint32_t)ldf * 4u;
                        }
                    }
                };
                if (C && F) emit(std::true_type{}, std::true_type{});
                else if (F) emit(std::false_type{}, std::true_type{});
                else emit(std::true_type{}, std::false_type{});
            }
            if (bits) {       // one ballot = 16 columns of four rows (lanes 16q .. 16q+15: row 4q + r); columns >= N give 0
                uint16_t* sh = reinterpret_cast<uint16_t*>(sb) + cur * TR * 8;
#pragma unroll
                for (int c = 0; c < NCW; ++c) {
                    const int cb = col_block(c);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const unsigned long long b = __ballot(acc[c][r] > 0.f);
                        if (l16 == 0 && cb < 8) sh[(16 * rowblk + 4 * lq + r) * 8 + cb] = (uint16_t)(b >> (16 * lq));
                    }
                }
            }
        }
        __syncthreads();
        cur ^= 1;
    }
    if (bits && prev >= 0) flush_bits(cur ^ 1, prev);                    // the last pass ended with a barrier
}

// ---- the small-width forward product through the bf16 matrix instructions ---------------------------
// Same persistent structure as k_gemm_small_f32, for the shapes whose fp32 matrix work binds (K and N
// above 32): every fp32 operand is split into three bf16 numbers (the row tile once, when it is
// written to LDS as three planes; the weights once, in registers) and six bf16 products replace one
// fp32 product (see split3).  A workgroup walks tiles of 64 rows; block q = w + 4t of the 2 x TNB grid
// of 32x32 blocks belongs to wavefront w, which therefore always works on column block w % TNB.
#ifndef PLX_X3_FWD_WAVES
#define PLX_X3_FWD_WAVES 2
#endif
#ifndef PLX_X3_FWD_CAP
#define PLX_X3_FWD_CAP 0
#endif
// NEXT: the tile of the result (activated if F is written) also goes to LDS in fp32 and is multiplied there by
// Wn[N x dn], dn <= 16: Tn[M x dn] = act(A B) Wn, the combine step (Eq. 2.2) of a following combine-first layer,
// which then does not read the M x N result back.  Wavefront w forms rows 16w .. 16w+15 of the tile's Tn with
// v_mfma_f32_16x16x4_f32 (lane l: a = tile[16w + l%16][4s + l/16], b = Wn[4s + l/16][l%16], in registers for the
// whole kernel; acc[r] = Tn[16w + 4*(l/16) + r][l%16]).
template <int TKB, int TNB, bool NEXT>   // 32 < K <= 32*TKB, 32 < N <= 32*TNB (TKB, TNB in {2, 4}); 16-byte aligned rows, K % 4 == 0
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(PLX_X3_FWD_WAVES))) void k_gemm_small_x3(int64_t M, int N, int K, const float* __restrict__ A,
                                                       int64_t lda, const float* __restrict__ B, int64_t ldb,
                                                       float* __restrict__ C, int64_t ldc, float* __restrict__ F,
                                                       int64_t ldf, uint32_t* __restrict__ bits, int64_t ldbits,
                                                       int bits_vec, const float* __restrict__ Wn, int64_t ldwn, int dn,
                                                       float* __restrict__ Tn, int64_t ldtn) {
    constexpr int KP = 32 * TKB, ROWS = 64, NBLK = 2 * TNB / 4, NKS = KP / 16, SA = KP + 8, PLANE = ROWS * SA;
    constexpr int NLD = ROWS * KP / 4 / 256;
    constexpr int NPC = 32 * TNB, FP = NPC + 4;                              // the fp32 copy of the result tile: [ROWS][FP]
    extern __shared__ __align__(16) unsigned char smem_raw[];
    bf16_t* As = reinterpret_cast<bf16_t*>(smem_raw);                        // [3][ROWS][SA]
    uint32_t* sb = reinterpret_cast<uint32_t*>(As + 3 * PLANE);              // sign bits: [2][4 words][ROWS]
    float* Ft = reinterpret_cast<float*>(sb + 2 * 4 * ROWS);                 // only with NEXT
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5;
    const int bj = w % TNB;

    bf16x8 breg[NKS][3];                   // planes of B[16s + 8*lh .. +7][32*bj + l32]
    {
        const int n = 32 * bj + l32;
#pragma unroll
        for (int s2 = 0; s2 < NKS; ++s2) {
            Frag f[3];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float x[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int kk = 16 * s2 + 8 * lh + 4 * h + e;
                    x[e] = (kk < K && n < N) ? B[(int64_t)kk * ldb + n] : 0.f;
                }
                uint2 pl[3];
                split3<true>(make_float4(x[0], x[1], x[2], x[3]), pl);
#pragma unroll
                for (int p = 0; p < 3; ++p) { f[p].x[2 * h] = pl[p].x; f[p].x[2 * h + 1] = pl[p].y; }
            }
#pragma unroll
            for (int p = 0; p < 3; ++p) breg[s2][p] = f[p].v;
        }
    }
    constexpr int NWS = NEXT ? NPC / 4 : 1;
    float wn[NWS];                         // wn[s] = Wn[4s + l/16][l%16]
    if constexpr (NEXT) {
        const int l16 = lane & 15, lq = lane >> 4;
#pragma unroll
        for (int s4 = 0; s4 < NWS; ++s4) {
            const int k = 4 * s4 + lq;
            wn[s4] = (k < N && l16 < dn) ? Wn[(int64_t)k * ldwn + l16] : 0.f;
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);    // weights landed before the row loop (vmcnt(0))

    const int64_t n_tiles = (M + ROWS - 1) / ROWS;
    float4 reg[NLD];
    uint32_t toff[NLD];                    // byte offset of a thread's 16-byte pieces inside a tile
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int f = tid + 256 * i, r = f / (KP / 4), q = f % (KP / 4);
        toff[i] = (KP == K || 4 * q < K) ? (uint32_t)(((uint32_t)r * (uint32_t)lda + 4u * q) * 4u) : kOutOfRange;
    }
    const uint32_t tile_bytes_a = (uint32_t)(((ROWS - 1) * lda + K) * 4);
    auto fetch = [&](int64_t tile) {       // the byte count ends with the last valid row: rows past it read as 0
        const int64_t m0 = tile * ROWS, left = M - m0;
        const __amdgpu_buffer_rsrc_t ra = buffer_of(A + m0 * lda, left >= ROWS ? tile_bytes_a : (uint32_t)(((left - 1) * lda + K) * 4));
#pragma unroll
        for (int i = 0; i < NLD; ++i) reg[i] = buffer_load4(ra, toff[i]);
    };
    auto commit = [&]() {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int f = tid + 256 * i, r = f / (KP / 4), q = f % (KP / 4);
            uint2 pl[3];
            split3(reg[i], pl);
#pragma unroll
            for (int p = 0; p < 3; ++p) *reinterpret_cast<uint2*>(As + p * PLANE + r * SA + 4 * q) = pl[p];
        }
    };
    const int nw = (N + 31) >> 5;
    auto flush_bits = [&](int buf, int64_t t) {                          // words of tile t, written by the pass before
        const int64_t row = t * ROWS + tid;
        if (tid < ROWS && row < M) {
            uint32_t wds[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) wds[j] = j < TNB ? sb[(buf * 4 + j) * ROWS + tid] : 0u;
            uint32_t* dst = bits + row * ldbits;
            if (bits_vec == 4) *reinterpret_cast<uint4*>(dst) = make_uint4(wds[0], wds[1], wds[2], wds[3]);
            else if (bits_vec == 2) *reinterpret_cast<uint2*>(dst) = make_uint2(wds[0], wds[1]);
            else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (j < nw) dst[j] = wds[j];
            }
        }
    };

    int64_t tile = blockIdx.x, prev = -1;
    int cur = 0;
    if (tile < n_tiles) { fetch(tile); commit(); }
    __syncthreads();
    const int k_end = (K + 15) & ~15;
    const uint32_t coff = (uint32_t)((4u * lh * (uint32_t)ldc + 32 * bj + l32) * 4u), foff = (uint32_t)((4u * lh * (uint32_t)ldf + 32 * bj + l32) * 4u);
    for (; tile < n_tiles; tile += gridDim.x) {
        fetch(tile + gridDim.x < n_tiles ? tile + gridDim.x : tile);     // unconditional: the last pass re-reads its own tile
        if (bits && prev >= 0) flush_bits(cur ^ 1, prev);
        prev = tile;
        floatx16 acc[NBLK];
#pragma unroll
        for (int t = 0; t < NBLK; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
#pragma unroll
        for (int s2 = 0; s2 < NKS; ++s2) {
            if (s2 > 0 && 16 * s2 >= k_end) break;                       // uniform
#pragma unroll
            for (int t = 0; t < NBLK; ++t) {
                const int bi = (w + 4 * t) / TNB;
                bf16x8 a[3];
#pragma unroll
                for (int p = 0; p < 3; ++p) a[p] = frag_contig(As + p * PLANE + (32 * bi + l32) * SA + 16 * s2 + 8 * lh);
                PLX_X3_32(acc[t], a, breg[s2]);
            }
        }
        if constexpr (NEXT) {                                            // what the following layer reads: act(result), columns >= N are 0
#pragma unroll
            for (int t = 0; t < NBLK; ++t) {
                const int bi = (w + 4 * t) / TNB;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float v = acc[t][r];
                    Ft[(32 * bi + 8 * (r / 4) + 4 * lh + (r % 4)) * FP + 32 * bj + l32] = F ? relu0(v) : v;
                }
            }
        }
        __syncthreads();                                                 // every wavefront is done reading the tile
        commit();
        const int64_t m0 = tile * ROWS;
        const bool full = m0 + ROWS <= M;                                // uniform: only the last tile is partial
        if (32 * bj + l32 < N) {
            const __amdgpu_buffer_rsrc_t rc = buffer_of(C ? C + m0 * ldc : nullptr, (uint32_t)(((ROWS - 1) * ldc + N) * 4));
            const __amdgpu_buffer_rsrc_t rf = buffer_of(F ? F + m0 * ldf : nullptr, (uint32_t)(((ROWS - 1) * ldf + N) * 4));
            auto emit = [&](auto guarded, auto has_c, auto has_f) {
#pragma unroll
                for (int t = 0; t < NBLK; ++t) {
                    const int bi = (w + 4 * t) / TNB;                    // uniform
                    uint32_t crow = opaque_zero() + 32u * bi * (uint32_t)ldc * 4u, frow = opaque_zero() + 32u * bi * (uint32_t)ldf * 4u;
                    int at = 0;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int row = 8 * (r / 4) + (r % 4);             // inside the block, of the lower half-wave
                        crow += (uint32_t)(row - at) * (uint32_t)ldc * 4u;
                        frow += (uint32_t)(row - at) * (uint32_t)ldf * 4u;
                        at = row;
                        const float v = acc[t][r];
                        if (!guarded.value || m0 + 32 * bi + row + 4 * lh < M) {
                            if (has_c.value) buffer_store_nt(rc, coff, crow, v);
                            if (has_f.value) buffer_store_nt(rf, foff, frow, relu0(v));   // Eq. 2.3 fused into the store
                        }
                    }
                }
            };
            auto emit_cf = [&](auto guarded) {
                if (C && F) emit(guarded, std::true_type{}, std::true_type{});
                else if (F) emit(guarded, std::false_type{}, std::true_type{});
                else emit(guarded, std::true_type{}, std::false_type{});
            };
            if (full) emit_cf(std::false_type{}); else emit_cf(std::true_type{});
        }
        if (bits) {       // one ballot = 32 columns of two rows (lanes 0-31: row dr, lanes 32-63: row dr + 4); columns >= N give 0
#pragma unroll
            for (int t = 0; t < NBLK; ++t) {
                const int bi = (w + 4 * t) / TNB;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    uint32_t lo[4], hi[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const unsigned long long b = __ballot(acc[t][4 * g + j] > 0.f);
                        lo[j] = (uint32_t)b;
                        hi[j] = (uint32_t)(b >> 32);
                    }
                    if (lane == 0) {
                        uint4* dst = reinterpret_cast<uint4*>(&sb[(cur * 4 + bj) * ROWS + 32 * bi + 8 * g]);
                        dst[0] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
                        dst[1] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
                    }
                }
            }
        }
        if constexpr (NEXT) {                                            // Tn rows 16w .. 16w+15 of this tile
            const int l16 = lane & 15, lq = lane >> 4;
            floatx4 tacc = floatx4{0.f, 0.f, 0.f, 0.f};
            const float* frow = Ft + (16 * w + l16) * FP + lq;
            const int n_end4 = (N + 3) / 4;
#pragma unroll
            for (int s4 = 0; s4 < NWS; ++s4) {
                if (s4 >= n_end4) break;                                 // uniform
                tacc = __builtin_amdgcn_mfma_f32_16x16x4f32(frow[4 * s4], wn[s4], tacc, 0, 0, 0);
            }
            if (l16 < dn) {
                const __amdgpu_buffer_rsrc_t rt = buffer_of(Tn + m0 * ldtn, (uint32_t)(((ROWS - 1) * ldtn + dn) * 4));
                const uint32_t toffs = (uint32_t)((4u * lq * (uint32_t)ldtn + l16) * 4u);
                uint32_t trow = opaque_zero() + 16u * w * (uint32_t)ldtn * 4u;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (full || m0 + 16 * w + 4 * lq + r < M) buffer_store(rt, toffs, trow, tacc[r]);
                    trow += (uint32_t)ldtn * 4u;
                }
            }
        }
        __syncthreads();
        cur ^= 1;
    }
    if (bits && prev >= 0) flush_bits(cur ^ 1, prev);                    // the last pass ended with a barrier
}

// ---- partial[chunk][M x N] = A[rows of chunk, M]^T * B[rows of chunk, N] ---------------------------
template <int TMB, int TNB>
__global__ __launch_bounds__(256) void k_gemm_tn_f32(int64_t R, int M, int N, const float* __restrict__ A, int64_t lda,
                                                     const float* __restrict__ B, int64_t ldb,
                                                     float* __restrict__ part, int64_t rows_per_chunk, int vec_a,
                                                     int vec_b) {
    constexpr int BM = 32 * TMB, BN = 32 * TNB;
    // NB output blocks over 4 wavefronts: NB >= 4 gives NB/4 blocks each; with NB < 4 the 4/NB
    // wavefronts that share a block take interleaved row pairs of every slab and write separate
    // partial tiles (slot = chunk * KS + slice), so no matrix instruction sits under a condition.
    constexpr int NB = TMB * TNB, KS = NB >= 4 ? 1 : 4 / NB, NBLK = NB >= 4 ? NB / 4 : 1;
    __shared__ __align__(16) float As[kBK][BM + 4];
    __shared__ __align__(16) float Bs[kBK][BN + 4];
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wq = NB >= 4 ? w : w % NB, ks = NB >= 4 ? 0 : w / NB;
    const int l32 = lane & 31, lh = lane >> 5;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.z * BN;
    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_chunk;
    const int64_t r_end = (r_begin + rows_per_chunk < R) ? r_begin + rows_per_chunk : R;

    floatx16 acc[NBLK];
#pragma unroll
    for (int t = 0; t < NBLK; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

    for (int64_t r0 = r_begin; r0 < r_end; r0 += kBK) {
        for (int f = tid; f < kBK * BM / 4; f += 256) {
            const int kk = f / (BM / 4), q = f % (BM / 4);
            const int64_t gr = r0 + kk;
            const int gm = m0 + 4 * q;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (gr < r_end) {
                const float* p = A + gr * lda + gm;
                if (vec_a && gm + 3 < M) {
                    v = *reinterpret_cast<const float4*>(p);
                } else {
                    if (gm < M) v.x = p[0];
                    if (gm + 1 < M) v.y = p[1];
                    if (gm + 2 < M) v.z = p[2];
                    if (gm + 3 < M) v.w = p[3];
                }
            }
            *reinterpret_cast<float4*>(&As[kk][4 * q]) = v;
        }
        for (int f = tid; f < kBK * BN / 4; f += 256) {
            const int kk = f / (BN / 4), q = f % (BN / 4);
            const int64_t gr = r0 + kk;
            const int gn = n0 + 4 * q;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (gr < r_end) {
                const float* p = B + gr * ldb + gn;
                if (vec_b && gn + 3 < N) {
                    v = *reinterpret_cast<const float4*>(p);
                } else {
                    if (gn < N) v.x = p[0];
                    if (gn + 1 < N) v.y = p[1];
                    if (gn + 2 < N) v.z = p[2];
                    if (gn + 3 < N) v.w = p[3];
                }
            }
            *reinterpret_cast<float4*>(&Bs[kk][4 * q]) = v;
        }
        __syncthreads();
#pragma unroll 4
        for (int kk = 2 * ks; kk < kBK; kk += 2 * KS) {
#pragma unroll
            for (int t = 0; t < NBLK; ++t) {
                const int q = wq + 4 * t, bi = q / TNB, bj = q % TNB;
                acc[t] = mfma32(As[kk + lh][32 * bi + l32], Bs[kk + lh][32 * bj + l32], acc[t]);
            }
        }
        __syncthreads();
    }
    float* out = part + ((int64_t)blockIdx.x * KS + ks) * M * N;
#pragma unroll
    for (int t = 0; t < NBLK; ++t) {
        const int q = wq + 4 * t, bi = q / TNB, bj = q % TNB;
        const int gn = n0 + 32 * bj + l32;
        if (gn >= N) continue;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int gm = m0 + 32 * bi + 8 * (r / 4) + 4 * lh + (r % 4);
            if (gm < M) out[(int64_t)gm * N + gn] = acc[t][r];
        }
    }
}

// The same partial products for 16-byte aligned operands: buffer loads with lane offsets computed
// once, the next slab of 32 rows in flight while the matrix cores work on the current one, two LDS
// buffers and one barrier per slab.  Block ownership, slot layout and summation order inside a
// chunk are those of the kernel above.  T = bf16_t: both operands hold bf16 and are widened on
// their way into LDS (exact); the partial sums and the result stay fp32.
template <int TMB, int TNB, typename T>
__global__ __launch_bounds__(256) void k_gemm_tn_deep(int64_t R, int M, int N, const T* __restrict__ A, int64_t lda,
                                                      const T* __restrict__ B, int64_t ldb,
                                                      float* __restrict__ part, int64_t rows_per_chunk) {
    constexpr int BM = 32 * TMB, BN = 32 * TNB, AP = BM + 4, BP = BN + 4;
    constexpr int NB = TMB * TNB, KS = NB >= 4 ? 1 : 4 / NB, NBLK = NB >= 4 ? NB / 4 : 1;
    constexpr int NE = RowPiece<T>::N;
    constexpr int PA = kBK * BM / NE, PB = kBK * BN / NE;               // 16-byte pieces of a slab: 128 (bf16, 32 wide) .. 1024
    constexpr int NA = (PA + 255) / 256, NBV = (PB + 255) / 256;        // per thread
    extern __shared__ __align__(16) float smem[];
    typedef float (*ATile)[AP];
    typedef float (*BTile)[BP];
    auto a_buf = [&](int b) { return reinterpret_cast<ATile>(smem + b * kBK * (AP + BP)); };
    auto b_buf = [&](int b) { return reinterpret_cast<BTile>(smem + b * kBK * (AP + BP) + kBK * AP); };
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wq = NB >= 4 ? w : w % NB, ks = NB >= 4 ? 0 : w / NB;
    const int l32 = lane & 31, lh = lane >> 5;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.z * BN;
    const int mcols = M - m0 < BM ? M - m0 : BM, ncols = N - n0 < BN ? N - n0 : BN;
    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_chunk;
    const int64_t r_end = (r_begin + rows_per_chunk < R) ? r_begin + rows_per_chunk : R;

    uint32_t offa[NA], offb[NBV];                  // threads beyond a slab's pieces (PA or PB = 128) load nothing and write nothing
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int f = tid + 256 * i, kk = f / (BM / NE), q = f % (BM / NE);
        offa[i] = f < PA ? ((uint32_t)kk * (uint32_t)lda + (uint32_t)(NE * q)) * (uint32_t)sizeof(T) : kOutOfRange;
    }
#pragma unroll
    for (int i = 0; i < NBV; ++i) {
        const int f = tid + 256 * i, kk = f / (BN / NE), q = f % (BN / NE);
        offb[i] = f < PB ? ((uint32_t)kk * (uint32_t)ldb + (uint32_t)(NE * q)) * (uint32_t)sizeof(T) : kOutOfRange;
    }
    float4 ra[NA], rb[NBV];
    auto fetch = [&](int64_t r0) {
        // byte counts end with the last valid element of the slab: rows past the chunk read as 0; columns past
        // M or N of the other rows hold whatever follows them in memory and only reach outputs that are not stored
        const int64_t left = r_end - r0;
        const int krows = (int)(left < kBK ? left : kBK);
        const __amdgpu_buffer_rsrc_t da = buffer_of(A + r0 * lda + m0, extent_bytes<T>(krows - 1, lda, mcols));
        const __amdgpu_buffer_rsrc_t db = buffer_of(B + r0 * ldb + n0, extent_bytes<T>(krows - 1, ldb, ncols));
#pragma unroll
        for (int i = 0; i < NA; ++i) ra[i] = buffer_load4(da, offa[i]);
#pragma unroll
        for (int i = 0; i < NBV; ++i) rb[i] = buffer_load4(db, offb[i]);
    };
    auto commit = [&](int b) {
        ATile As = a_buf(b);
        BTile Bs = b_buf(b);
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int f = tid + 256 * i;
            float4 v[NE / 4];
            RowPiece<T>::widen(ra[i], v);
            if (PA % 256 == 0 || f < PA) {
#pragma unroll
                for (int j = 0; j < NE / 4; ++j) *reinterpret_cast<float4*>(&As[f / (BM / NE)][NE * (f % (BM / NE)) + 4 * j]) = v[j];
            }
        }
#pragma unroll
        for (int i = 0; i < NBV; ++i) {
            const int f = tid + 256 * i;
            float4 v[NE / 4];
            RowPiece<T>::widen(rb[i], v);
            if (PB % 256 == 0 || f < PB) {
#pragma unroll
                for (int j = 0; j < NE / 4; ++j) *reinterpret_cast<float4*>(&Bs[f / (BN / NE)][NE * (f % (BN / NE)) + 4 * j]) = v[j];
            }
        }
    };

    floatx16 acc[NBLK];
#pragma unroll
    for (int t = 0; t < NBLK; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

    if (r_begin < r_end) {                         // uniform
        fetch(r_begin);
        commit(0);
    }
    __syncthreads();
    int cur = 0;
    for (int64_t r0 = r_begin; r0 < r_end; r0 += kBK) {
        fetch(r0 + kBK < r_end ? r0 + kBK : r0);   // no condition around the prefetch: the last pass re-reads its own slab
        ATile As = a_buf(cur);
        BTile Bs = b_buf(cur);
#pragma unroll
        for (int kk = 2 * ks; kk < kBK; kk += 2 * KS) {
            float a[NBLK], b[NBLK];
#pragma unroll
            for (int t = 0; t < NBLK; ++t) {
                const int q = wq + 4 * t, bi = q / TNB, bj = q % TNB;
                a[t] = As[kk + lh][32 * bi + l32];
                b[t] = Bs[kk + lh][32 * bj + l32];
            }
#pragma unroll
            for (int t = 0; t < NBLK; ++t) acc[t] = mfma32(a[t], b[t], acc[t]);
        }
        commit(cur ^ 1);                           // the barrier of the pass before ended every read of that buffer
        __syncthreads();
        cur ^= 1;
    }
    float* out = part + ((int64_t)blockIdx.x * KS + ks) * M * N;
#pragma unroll
    for (int t = 0; t < NBLK; ++t) {
        const int q = wq + 4 * t, bi = q / TNB, bj = q % TNB;
        const int gn = n0 + 32 * bj + l32;
        if (gn >= N) continue;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int gm = m0 + 32 * bi + 8 * (r / 4) + 4 * lh + (r % 4);
            if (gm < M) out[(int64_t)gm * N + gn] = acc[t][r];
        }
    }
}

// One level of the fixed-order sum of partial tiles: slot g*kFan*stride receives the sum of the
// live slots (g*kFan + t)*stride, t = 0..kFan-1.  With `final_out` the sums go to C instead.
constexpr int kFan = 32;
__global__ __launch_bounds__(256) void k_reduce_partials(float* __restrict__ part, int64_t elems, int64_t n_live,
                                                         int64_t stride, float* __restrict__ C, int N, int64_t ldc) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t g = blockIdx.y;
    if (e >= elems) return;
    float s = 0.f;
    for (int t = 0; t < kFan; ++t) {
        const int64_t slot = g * kFan + t;
        if (slot >= n_live) break;
        s += part[slot * stride * elems + e];
    }
    if (C) C[(e / N) * ldc + (e % N)] = s;
    else part[g * kFan * stride * elems + e] = s;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

int64_t tn_rows_per_chunk(int64_t R, int64_t M, int64_t N) {
    const int64_t tiles = ceil_div(M, 128) * ceil_div(N, 128);
    const int64_t want_chunks = std::max<int64_t>(1, 2048 / tiles);     // measured flat between 2048 and 16384
    // a chunk's partial tile costs a write and a read of M x N floats: chunks keep at least 512 rows
    // unless the matrix is so short that this would leave most CUs without work
    const int64_t min_rows = std::min<int64_t>(512, std::max<int64_t>(64, R / 1024));
    int64_t rows = std::max<int64_t>(min_rows, ceil_div(R, want_chunks));
    return ceil_div(rows, 64) * 64;
}

// fixed-order tree over `chunks` partial M x N tiles; the total goes to C
plx_status reduce_partials(plx_ctx* ctx, float* part, int64_t chunks, int64_t M, int64_t N, float* C, int64_t ldc) {
    KernelTimer kt(ctx, "dw_partials_reduce");
    const int64_t elems = M * N;
    int64_t live = chunks, stride = 1;
    while (true) {
        const int64_t groups = ceil_div(live, kFan);
        const bool last = groups == 1;
        dim3 rgrid((unsigned)ceil_div(elems, 256), (unsigned)groups);
        k_reduce_partials<<<rgrid, 256, 0, ctx->stream>>>(part, elems, live, stride, last ? C : nullptr, (int)N, ldc);
        if (last) break;
        live = groups;
        stride *= kFan;
    }
    PLX_HIP(ctx, hipGetLastError());
    return PLX_OK;
}

// wavefronts sharing one output block (see the kernels): 4 / (number of 32x32 blocks) when that is < 4
int tn_kslices(int64_t M, int64_t N) {
    const int tmb = M <= 32 ? 1 : (M <= 64 ? 2 : 4), tnb = N <= 32 ? 1 : (N <= 64 ? 2 : 4);
    return tmb * tnb >= 4 ? 1 : 4 / (tmb * tnb);
}

size_t gemm_tn_workspace(int64_t R, int64_t M, int64_t N) {
    const int64_t chunks = std::max<int64_t>(1, ceil_div(R, tn_rows_per_chunk(R, M, N)));
    return (size_t)chunks * tn_kslices(M, N) * (size_t)M * (size_t)N * sizeof(float);
}

namespace {

// what the slab kernels need: 16-byte aligned rows (the lane offsets are 16-byte pieces) and tiles whose byte
// offsets fit 31 bits (128 rows of up to 2^22 elements)
bool deep_operand(const void* p, int64_t ld, plx_dtype dtype) {
    return aligned16(p) && ld % (16 / (int64_t)elt_size(dtype)) == 0 && ld < (int64_t(1) << 22);
}

template <int TNB, bool BT, typename TA>
auto gemm_deep_kernel(bool bv) { return bv ? k_gemm_deep<TNB, BT, TA, true> : k_gemm_deep<TNB, BT, TA, false>; }

template <typename TA>
plx_status launch_gemm_deep(plx_ctx* ctx, bool bt, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const float* B,
                            int64_t ldb, void* C, int64_t ldc, void* Fact, int64_t ldf) {
    const int tnb = N <= 32 ? 1 : (N <= 64 ? 2 : 4);
    const dim3 grid((unsigned)ceil_div(M, 128), (unsigned)ceil_div(N, 32 * tnb));
    const size_t lds_b = bt ? 32 * tnb * (kBK + 4) : kBK * (32 * tnb + 4);
    const size_t lds = sizeof(float) * 2 * (128 * (kBK + 4) + lds_b);
    auto launch = [&](auto kern) -> plx_status {
        if (lds > 48 * 1024)
            PLX_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        kern<<<grid, 256, lds, ctx->stream>>>(M, (int)N, (int)K, static_cast<const TA*>(A), lda, B, ldb, static_cast<TA*>(C), ldc,
                                              static_cast<TA*>(Fact), ldf);
        PLX_HIP(ctx, hipGetLastError());
        return PLX_OK;
    };
    const bool bv = aligned16(B) && ldb % 4 == 0;      // the weight matrix may have rows of any length (41, 47 classes)
    if (bt) {
        if (tnb == 1) return launch(gemm_deep_kernel<1, true, TA>(bv));
        if (tnb == 2) return launch(gemm_deep_kernel<2, true, TA>(bv));
        return launch(gemm_deep_kernel<4, true, TA>(bv));
    }
    if (tnb == 1) return launch(gemm_deep_kernel<1, false, TA>(bv));
    if (tnb == 2) return launch(gemm_deep_kernel<2, false, TA>(bv));
    return launch(gemm_deep_kernel<4, false, TA>(bv));
}

}  // namespace

// Does the nn product of these shapes go through the split kernel, which can multiply its result tile by a
// following layer's Wn[N x dn] on the way out?
bool gemm_next_supported(const plx_ctx* ctx, int64_t M, int64_t N, int64_t K, int64_t dn, plx_dtype dtype, const void* A, int64_t lda,
                         int64_t ldc, int64_t ldf, int64_t ldtn) {
    const int64_t cap = int64_t(1) << 23;
    return dtype == PLX_F32 && ctx->split_products && M > 0 && K > 32 && K <= 128 && N > 32 && N <= 128 && K % 4 == 0 && dn > 0 &&
           dn <= 16 && aligned16(A) && lda % 4 == 0 && lda < cap && ldc < cap && ldf < cap && ldtn < cap;
}

plx_status launch_gemm(plx_ctx* ctx, bool bt, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                       const float* B, int64_t ldb, void* C, int64_t ldc, plx_dtype dtype, void* Fact, int64_t ldf,
                       uint32_t* bits, int64_t ldbits, const float* Wn, int64_t ldwn, int64_t dn, float* Tn, int64_t ldtn) {
    if (bits && !Fact) return fail(ctx, PLX_ERR_INTERNAL, "sign bits are written next to the activated output");
    if (Tn && (bt || !gemm_next_supported(ctx, M, N, K, dn, dtype, A, lda, C ? ldc : 0, Fact ? ldf : 0, ldtn)))
        return fail(ctx, PLX_ERR_INTERNAL, "chained product outside the split kernel's range");
    if (N >= (int64_t(1) << 20) || K >= (int64_t(1) << 30)) return fail(ctx, PLX_ERR_UNSUPPORTED, "N or K too large");
    const bool deep = M > 0 && N > 0 && K > 0 && deep_operand(A, lda, dtype) && ldb < (int64_t(1) << 22) &&
                      (!C || ldc < (int64_t(1) << 22)) && (!Fact || ldf < (int64_t(1) << 22));
    if (dtype == PLX_BF16) {
        if (!bt && K <= 128 && N <= 128) return launch_gemm_small_bf16(ctx, M, N, K, A, lda, B, ldb, C, ldc, Fact, ldf, bits, ldbits);
        // wider layers (and A B^T outside the fused backward kernel): the slab kernel, bf16 widened on load
        if (!deep)
            return fail(ctx, PLX_ERR_UNSUPPORTED, "bf16 products with K or N above 128, and A B^T, need 16-byte aligned rows of A (lda %% 8 == 0) and leading dimensions below 2^22 elements");
        char label[64];
        snprintf(label, sizeof label, "gemm_%s<bf16>[M%lld,N%lld,K%lld]w32", bt ? "nt" : "nn", (long long)M, (long long)N, (long long)K);
        {
            KernelTimer kt(ctx, label);
            PLX_TRY(launch_gemm_deep<bf16_t>(ctx, bt, M, N, K, A, lda, B, ldb, C, ldc, Fact, ldf));
        }
        if (bits) return launch_bits_from_act(ctx, M, N, Fact, ldf, bits, ldbits, dtype);
        return PLX_OK;
    }
    const float* a = static_cast<const float*>(A);
    float* c = static_cast<float*>(C);
    float* fa = static_cast<float*>(Fact);
    const int vec_a = aligned16(A) && lda % 4 == 0;
    const int tnb = N <= 32 ? 1 : (N <= 64 ? 2 : 4);
    dim3 grid((unsigned)ceil_div(M, 128), (unsigned)ceil_div(N, 32 * tnb));
    hipStream_t s = ctx->stream;
    // the small-width kernels address a tile with 31-bit byte offsets: 64 rows * ld * 4 bytes must fit
    const bool ld32 = lda < (int64_t(1) << 23) && (!C || ldc < (int64_t(1) << 23)) && (!Fact || ldf < (int64_t(1) << 23));
    const bool small = !bt && K <= 128 && N <= 128 && K > 0 && ld32;
    // K and N above 32: the fp32 matrix pipe would bind, six bf16 products per fp32 product are taken instead
    const bool split = small && ctx->split_products && vec_a && K % 4 == 0 && M > 0 && K > 32 && N > 32;
    char label[64];
    char next[16] = "";
    if (Tn) snprintf(next, sizeof next, "next%lld", (long long)dn);    // also multiplies its result by the following layer's weights
    snprintf(label, sizeof label, "gemm_%s<f32>[M%lld,N%lld,K%lld]%s%s", bt ? "nt" : "nn", (long long)M, (long long)N, (long long)K,
             split ? "x3" : "", next);
    KernelTimer kt(ctx, label);
    if (small) {
        const int tkb = K <= 32 ? 1 : (K <= 64 ? 2 : 4);
        int cb = (int)ceil_div(N, 16);
        if (cb > 4) cb = 8;                    // wide tiles are 128 columns (four 32x32 column blocks)
        const int tr = fwd_tile_rows(tkb, cb);
        const size_t lds = sizeof(float) * 2 * tr * (32 * tkb + 4) + (bits ? 2 * tr * 16 : 0);
        const bool vec = vec_a && K % 4 == 0 && M > 0;
        const int nw = (int)ceil_div(N, 32);
        const uintptr_t bp = reinterpret_cast<uintptr_t>(bits);
        const int bits_vec = (nw == 4 && ldbits % 4 == 0 && bp % 16 == 0) ? 4 : ((nw == 2 && ldbits % 2 == 0 && bp % 8 == 0) ? 2 : 1);
        if (split) {
            const int tnb3 = N <= 64 ? 2 : 4;
            const size_t lds3 = sizeof(uint16_t) * 3 * 64 * (32 * tkb + 8) + ((bits || Tn) ? 2 * 4 * 64 * 4 : 0) +
                                (Tn ? sizeof(float) * 64 * (32 * tnb3 + 4) : 0);
            auto launch_x3 = [&](auto kern) -> plx_status {
                if (lds3 > 48 * 1024)
                    PLX_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds3));
                int per_cu = 0;
                PLX_HIP(ctx, hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, 256, lds3));
                if (PLX_X3_FWD_CAP > 0) per_cu = std::min(per_cu, PLX_X3_FWD_CAP);
                const int64_t blocks = std::min<int64_t>(ceil_div(M, 64), (int64_t)ctx->n_cu * std::max(1, per_cu));
                kern<<<dim3((unsigned)blocks), 256, lds3, s>>>(M, (int)N, (int)K, a, lda, B, ldb, c, ldc, fa, ldf, bits, ldbits, bits_vec,
                                                               Wn, ldwn, (int)dn, Tn, ldtn);
                PLX_HIP(ctx, hipGetLastError());
                return PLX_OK;
            };
            if (Tn) {
                if (tkb == 2) return tnb3 == 2 ? launch_x3(k_gemm_small_x3<2, 2, true>) : launch_x3(k_gemm_small_x3<2, 4, true>);
                return tnb3 == 2 ? launch_x3(k_gemm_small_x3<4, 2, true>) : launch_x3(k_gemm_small_x3<4, 4, true>);
            }
            if (tkb == 2) return tnb3 == 2 ? launch_x3(k_gemm_small_x3<2, 2, false>) : launch_x3(k_gemm_small_x3<2, 4, false>);
            return tnb3 == 2 ? launch_x3(k_gemm_small_x3<4, 2, false>) : launch_x3(k_gemm_small_x3<4, 4, false>);
        }
        auto launch_small = [&](auto kern) -> plx_status {
            if (lds > 48 * 1024)
                PLX_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            int per_cu = 0;                    // resident workgroups per CU for this kernel's registers and LDS
            PLX_HIP(ctx, hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, 256, lds));
#ifndef PLX_FWD_WIDE_CAP_K32
#define PLX_FWD_WIDE_CAP_K32 2
#endif
            // measured: the store-bound K <= 32 case is fastest with 2 resident workgroups per CU (3: +4 %, 4: +8 %),
            // the matrix-bound K >= 64 cases with as many as fit (4)
            if (cb > 4 && tkb == 1) per_cu = std::min(per_cu, PLX_FWD_WIDE_CAP_K32);
            const int64_t blocks = std::min<int64_t>(ceil_div(M, tr), (int64_t)ctx->n_cu * std::max(1, per_cu));
            kern<<<dim3((unsigned)blocks), 256, lds, s>>>(M, (int)N, (int)K, a, lda, B, ldb, c, ldc, fa, ldf, bits, ldbits, bits_vec);
            return PLX_OK;
        };
#define PLX_SMALL(TK, CBV) \
    PLX_TRY(vec ? launch_small(k_gemm_small_f32<TK, CBV, true>) : launch_small(k_gemm_small_f32<TK, CBV, false>))
#define PLX_SMALL_K(CBV)                                         \
    do {                                                         \
        if (tkb == 1) PLX_SMALL(1, CBV);                         \
        else if (tkb == 2) PLX_SMALL(2, CBV);                    \
        else PLX_SMALL(4, CBV);                                  \
    } while (0)
        switch (cb) {
            case 1: PLX_SMALL_K(1); break;
            case 2: PLX_SMALL_K(2); break;
            case 3: PLX_SMALL_K(3); break;
            case 4: PLX_SMALL_K(4); break;
            default: PLX_SMALL_K(8); break;
        }
#undef PLX_SMALL_K
#undef PLX_SMALL
        PLX_HIP(ctx, hipGetLastError());
        return PLX_OK;
    }
    if (deep) {        // 16-byte aligned operands: the buffer-addressed slab kernel
        PLX_TRY(launch_gemm_deep<float>(ctx, bt, M, N, K, A, lda, B, ldb, C, ldc, Fact, ldf));
        if (bits) return launch_bits_from_act(ctx, M, N, Fact, ldf, bits, ldbits, dtype);
        return PLX_OK;
    }
#define PLX_GEMM_CASE(T, BTV) \
    k_gemm_f32<T, BTV><<<grid, 256, 0, s>>>(M, (int)N, (int)K, a, lda, B, ldb, c, ldc, fa, ldf, vec_a)
    if (bt) {
        if (tnb == 1) PLX_GEMM_CASE(1, true); else if (tnb == 2) PLX_GEMM_CASE(2, true); else PLX_GEMM_CASE(4, true);
    } else {
        if (tnb == 1) PLX_GEMM_CASE(1, false); else if (tnb == 2) PLX_GEMM_CASE(2, false); else PLX_GEMM_CASE(4, false);
    }
#undef PLX_GEMM_CASE
    PLX_HIP(ctx, hipGetLastError());
    if (bits) return launch_bits_from_act(ctx, M, N, Fact, ldf, bits, ldbits, dtype);    // no fused epilogue in the general kernel
    return PLX_OK;
}

plx_status launch_gemm_tn(plx_ctx* ctx, int64_t R, int64_t M, int64_t N, const void* A, int64_t lda, const void* B,
                          int64_t ldb, float* C, int64_t ldc, plx_dtype dtype, void* ws, size_t ws_bytes) {
    if (dtype == PLX_BF16 && M <= 128 && N <= 128)   // the fused kernel without its second product and without a mask
        return launch_bwd_dense_bf16(ctx, R, M, N, A, lda, B, ldb, nullptr, 0, nullptr, 0, nullptr, 0, C, ldc, ws, ws_bytes);
    if (M >= (int64_t(1) << 20) || N >= (int64_t(1) << 20)) return fail(ctx, PLX_ERR_UNSUPPORTED, "M or N too large");
    if (ws_bytes < gemm_tn_workspace(R, M, N)) return fail(ctx, PLX_ERR_SHAPE, "workspace too small");
    float* part = static_cast<float*>(ws);
    const int64_t rpc = tn_rows_per_chunk(R, M, N);
    const int64_t chunks = std::max<int64_t>(1, ceil_div(R, rpc));
    // 16-byte aligned operands whose 32-row slabs fit 31-bit byte offsets take the buffer-addressed kernel
    const bool deep = deep_operand(A, lda, dtype) && deep_operand(B, ldb, dtype);
    if (dtype == PLX_BF16 && !deep)
        return fail(ctx, PLX_ERR_UNSUPPORTED, "bf16 A^T B with M or N above 128 needs 16-byte aligned rows (ld %% 8 == 0) below 2^22 elements");
    const int vec_a = aligned16(A) && lda % 4 == 0, vec_b = aligned16(B) && ldb % 4 == 0;
    const int tmb = M <= 32 ? 1 : (M <= 64 ? 2 : 4);
    const int tnb = N <= 32 ? 1 : (N <= 64 ? 2 : 4);
    dim3 grid((unsigned)chunks, (unsigned)ceil_div(M, 32 * tmb), (unsigned)ceil_div(N, 32 * tnb));
    hipStream_t s = ctx->stream;
    char label[64];
    snprintf(label, sizeof label, "gemm_tn<%s>[R%lld,M%lld,N%lld]%s", dtype == PLX_BF16 ? "bf16" : "f32", (long long)R, (long long)M,
             (long long)N, dtype == PLX_BF16 ? "w32" : "");
    KernelTimer* kt = new KernelTimer(ctx, label);
    const size_t lds = deep ? sizeof(float) * 2 * kBK * (32 * tmb + 4 + 32 * tnb + 4) : 0;
    auto launch_deep = [&](auto kern, auto elt) -> hipError_t {
        typedef decltype(elt) T;
        if (lds > 48 * 1024) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        kern<<<grid, 256, lds, s>>>(R, (int)M, (int)N, static_cast<const T*>(A), lda, static_cast<const T*>(B), ldb, part, rpc);
        return hipSuccess;
    };
    hipError_t attr_err = hipSuccess;
#define PLX_TN_CASE(TM, TN)                                                                                  \
    do {                                                                                                     \
        if (dtype == PLX_BF16) attr_err = launch_deep(k_gemm_tn_deep<TM, TN, bf16_t>, bf16_t{});             \
        else if (deep) attr_err = launch_deep(k_gemm_tn_deep<TM, TN, float>, float{});                       \
        else                                                                                                 \
            k_gemm_tn_f32<TM, TN><<<grid, 256, 0, s>>>(R, (int)M, (int)N, static_cast<const float*>(A), lda, \
                                                       static_cast<const float*>(B), ldb, part, rpc, vec_a, vec_b); \
    } while (0)
    switch (tmb * 10 + tnb) {
        case 11: PLX_TN_CASE(1, 1); break;
        case 12: PLX_TN_CASE(1, 2); break;
        case 14: PLX_TN_CASE(1, 4); break;
        case 21: PLX_TN_CASE(2, 1); break;
        case 22: PLX_TN_CASE(2, 2); break;
        case 24: PLX_TN_CASE(2, 4); break;
        case 41: PLX_TN_CASE(4, 1); break;
        case 42: PLX_TN_CASE(4, 2); break;
        default: PLX_TN_CASE(4, 4); break;
    }
#undef PLX_TN_CASE
    delete kt;
    PLX_HIP(ctx, attr_err);
    PLX_HIP(ctx, hipGetLastError());
    return reduce_partials(ctx, part, chunks * tn_kslices(M, N), M, N, C, ldc);
}

}  // namespace plx
