// Dense products of a GCN layer with bf16 storage and fp32 accumulation (Eq. 2.2, 2.3 forward;
// Eq. 2.4, 2.5, 2.6 fused backward), for widths up to 128.  Activations and gradients are bf16 in
// HBM, the weight matrix is fp32 in HBM and rounded to bf16 (nearest even) when it is staged in
// LDS, products are exact in fp32 and accumulated in fp32 by v_mfma_f32_32x32x16_bf16 /
// v_mfma_f32_16x16x32_bf16.  At these widths the matrix work is a few percent of the time: the
// kernels are streaming kernels bound by HBM, organised like their fp32 counterparts (persistent
// workgroups, weights resident in LDS, next tile prefetched into registers during the MFMAs).
//
// Operand convention of both instructions: lane l supplies 8 consecutive k-values of row/column
// (l % 32 or l % 16), the k-slab chosen by l / 32 (or l / 16).  Both operands are fed with the
// same slab mapping, so the contraction is over all k whatever the hardware's numbering.
// Accumulator layouts equal those of the fp32 instructions of the same tile shape.
#include "plx_internal.h"

#include <algorithm>

namespace plx {
namespace {

typedef uint16_t bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

union Frag {
    uint4 u;
    bf16x8 v;
    bf16_t e[8];
};

__device__ __forceinline__ bf16_t f32_to_bf16(float f) {   // round to nearest even
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ bool bf16_positive(bf16_t z) { return (z & 0x8000u) == 0 && (z & 0x7fffu) != 0 && (z & 0x7fffu) <= 0x7f80u; }

// 8 consecutive bf16 of one row (16 bytes)
__device__ __forceinline__ bf16x8 frag_contig(const bf16_t* p) {
    Frag f;
    f.u = *reinterpret_cast<const uint4*>(p);
    return f.v;
}
// 8 bf16 one row apart each (a column of a row-major tile)
__device__ __forceinline__ bf16x8 frag_strided(const bf16_t* p, int stride) {
    Frag f;
#pragma unroll
    for (int i = 0; i < 8; ++i) f.e[i] = p[i * stride];
    return f.v;
}

// guarded load of 8 consecutive bf16 of a global row (zero beyond ncols / the last row)
__device__ __forceinline__ uint4 load8(const bf16_t* __restrict__ src, int64_t ld, int64_t gr, int64_t r_end, int gc,
                                       int ncols, bool vec) {
    Frag f;
    f.u = make_uint4(0, 0, 0, 0);
    if (gr < r_end && gc < ncols) {
        const bf16_t* p = src + gr * ld + gc;
        if (vec && gc + 7 < ncols) {
            f.u = *reinterpret_cast<const uint4*>(p);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (gc + i < ncols) f.e[i] = p[i];
        }
    }
    return f.u;
}

// ---- forward: C[M x N] = A[M x K] W[K x N] (+ ReLU copy), K, N <= 128 --------------------------------
template <int TKB, int TNB, int RB>
__global__ __launch_bounds__(256) void k_gemm_small_bf16(int64_t M, int N, int K, const bf16_t* __restrict__ A,
                                                         int64_t lda, const float* __restrict__ W, int64_t ldw,
                                                         bf16_t* __restrict__ C, int64_t ldc, bf16_t* __restrict__ F,
                                                         int64_t ldf, int vec_a) {
    constexpr int KP = 32 * TKB, NP = 32 * TNB, ROWS = 32 * RB;
    constexpr int NBLK = RB * TNB / 4;
    constexpr int NLD = (ROWS * KP / 8 + 255) / 256;       // 16-byte pieces per thread per tile
    constexpr int SA = KP + 8;                              // LDS row pitch in elements (16-byte multiple)
    static_assert((RB * TNB) % 4 == 0, "tile must split evenly over 4 wavefronts");
    extern __shared__ __align__(16) unsigned char smem_raw[];
    bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
    auto a_buf = [&](int b) { return smem + b * ROWS * SA; };
    bf16_t* Wt = smem + 2 * ROWS * SA;                      // W transposed: Wt[n][k]
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5;

    for (int f = tid; f < KP * NP; f += 256) {
        const int kk = f / NP, n = f % NP;
        Wt[n * SA + kk] = (kk < K && n < N) ? f32_to_bf16(W[(int64_t)kk * ldw + n]) : (bf16_t)0;
    }

    const int64_t n_tiles = (M + ROWS - 1) / ROWS;
    uint4 reg[NLD];
    auto fetch = [&](int64_t tile) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int f = tid + 256 * i, r = f / (KP / 8), q = f % (KP / 8);
            reg[i] = (f < ROWS * KP / 8) ? load8(A, lda, tile * ROWS + r, M, 8 * q, K, vec_a) : make_uint4(0, 0, 0, 0);
        }
    };
    auto commit = [&](bf16_t* As) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int f = tid + 256 * i, r = f / (KP / 8), q = f % (KP / 8);
            if (f < ROWS * KP / 8) *reinterpret_cast<uint4*>(As + r * SA + 8 * q) = reg[i];
        }
    };

    int64_t tile = blockIdx.x;
    int cur = 0;
    if (tile < n_tiles) { fetch(tile); commit(a_buf(0)); }
    __syncthreads();
    for (; tile < n_tiles; tile += gridDim.x) {
        // unconditional prefetch (the last pass re-reads its own tile): straight-line code keeps the
        // only wait for loads right before the LDS write
        fetch(tile + gridDim.x < n_tiles ? tile + gridDim.x : tile);
        const bf16_t* As = a_buf(cur);
        floatx16 acc[NBLK];
#pragma unroll
        for (int t = 0; t < NBLK; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KP; kk += 16) {
#pragma unroll
            for (int t = 0; t < NBLK; ++t) {
                const int q = w + 4 * t, bi = q / TNB, bj = q % TNB;
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_contig(As + (32 * bi + l32) * SA + kk + 8 * lh),
                                                                 frag_contig(Wt + (32 * bj + l32) * SA + kk + 8 * lh),
                                                                 acc[t], 0, 0, 0);
            }
        }
        commit(a_buf(cur ^ 1));
        const int64_t m0 = tile * ROWS;
#pragma unroll
        for (int t = 0; t < NBLK; ++t) {
            const int q = w + 4 * t, bi = q / TNB, bj = q % TNB;
            const int gn = 32 * bj + l32;
            if (gn >= N) continue;
            const int64_t row0 = m0 + 32 * bi + 4 * lh;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int dr = 8 * (r / 4) + (r % 4);
                if (row0 + dr < M) {
                    const float v = acc[t][r];
                    if (C) C[(row0 + dr) * ldc + gn] = f32_to_bf16(v);
                    if (F) F[(row0 + dr) * ldf + gn] = f32_to_bf16(v > 0.f ? v : 0.f);   // Eq. 2.3
                }
            }
        }
        __syncthreads();
        cur ^= 1;
    }
}

// ---- backward: dOut = (Q*[Zm>0]) W^T, dW partial = P^T (Q*[Zm>0]) ---------------------------------------
constexpr int kTR = 64;

template <int TMB, int TNB, bool MASK>
__global__ __launch_bounds__(256) void k_bwd_dense_bf16(int64_t R, int Mp, int N, const bf16_t* __restrict__ P,
                                                        int64_t ldp, const bf16_t* __restrict__ Q, int64_t ldq,
                                                        const bf16_t* __restrict__ Zm, int64_t ldz,
                                                        const float* __restrict__ W, int64_t ldw,
                                                        bf16_t* __restrict__ dOut, int64_t ldo, float* __restrict__ part,
                                                        int64_t rows_per_chunk, int vec_p, int vec_q) {
    constexpr int MP = 32 * TMB, NP = 32 * TNB, SQ = NP + 8, SP = MP + 8;
    constexpr int NB = TMB * TNB, KS = NB >= 4 ? 1 : 4 / NB, NBLK = NB >= 4 ? NB / 4 : 1;
    constexpr int NCB = MP / 16;
    constexpr int NQ = kTR * NP / 8 / 256, NPR = (kTR * MP / 8 + 255) / 256;   // 16-byte pieces per thread
    extern __shared__ __align__(16) unsigned char smem_raw[];
    bf16_t* Qs = reinterpret_cast<bf16_t*>(smem_raw);
    bf16_t* Ps = Qs + kTR * SQ;
    bf16_t* Ws = Ps + kTR * SP;                             // W as stored: Ws[i][n]
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5, l16 = lane & 15, lq = lane >> 4;
    const int wq = NB >= 4 ? w : w % NB, ks = NB >= 4 ? 0 : w / NB;
    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_chunk;
    const int64_t r_end = (r_begin + rows_per_chunk < R) ? r_begin + rows_per_chunk : R;

    for (int f = tid; f < MP * NP; f += 256) {
        const int i = f / NP, n = f % NP;
        Ws[i * SQ + n] = (W && i < Mp && n < N) ? f32_to_bf16(W[(int64_t)i * ldw + n]) : (bf16_t)0;
    }

    floatx16 acc_w[NBLK];
#pragma unroll
    for (int t = 0; t < NBLK; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_w[t][r] = 0.f;

    uint4 rq[NQ], rz[NQ], rp[NPR];
    auto fetch = [&](int64_t r0) {
#pragma unroll
        for (int i = 0; i < NQ; ++i) {
            const int f = tid + 256 * i, r = f / (NP / 8), q = f % (NP / 8);
            rq[i] = load8(Q, ldq, r0 + r, r_end, 8 * q, N, vec_q);
            if (MASK) rz[i] = load8(Zm, ldz, r0 + r, r_end, 8 * q, N, vec_q);
        }
#pragma unroll
        for (int i = 0; i < NPR; ++i) {
            const int f = tid + 256 * i, r = f / (MP / 8), q = f % (MP / 8);
            rp[i] = (f < kTR * MP / 8) ? load8(P, ldp, r0 + r, r_end, 8 * q, Mp, vec_p) : make_uint4(0, 0, 0, 0);
        }
    };
    auto commit = [&]() {
#pragma unroll
        for (int i = 0; i < NQ; ++i) {
            const int f = tid + 256 * i, r = f / (NP / 8), q = f % (NP / 8);
            Frag v;
            v.u = rq[i];
            if (MASK) {                                              // Eq. 2.4
                Frag z;
                z.u = rz[i];
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (!bf16_positive(z.e[e])) v.e[e] = 0;
            }
            *reinterpret_cast<uint4*>(Qs + r * SQ + 8 * q) = v.u;
        }
#pragma unroll
        for (int i = 0; i < NPR; ++i) {
            const int f = tid + 256 * i, r = f / (MP / 8), q = f % (MP / 8);
            if (f < kTR * MP / 8) *reinterpret_cast<uint4*>(Ps + r * SP + 8 * q) = rp[i];
        }
    };

    fetch(r_begin);
    commit();
    __syncthreads();
    for (int64_t r0 = r_begin; r0 < r_end; r0 += kTR) {
        fetch(r0 + kTR < r_end ? r0 + kTR : r0);      // unconditional, as in the forward kernel

        floatx4 acc_o[NCB];
        if (dOut) {                                                  // Eq. 2.6: wavefront w owns rows 16w..16w+15
#pragma unroll
            for (int c = 0; c < NCB; ++c) acc_o[c] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int k = 0; k < NP; k += 32) {
                const bf16x8 a = frag_contig(Qs + (16 * w + l16) * SQ + k + 8 * lq);
#pragma unroll
                for (int c = 0; c < NCB; ++c)
                    acc_o[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, frag_contig(Ws + (16 * c + l16) * SQ + k + 8 * lq),
                                                                       acc_o[c], 0, 0, 0);
            }
        }
#pragma unroll
        for (int kk = 16 * ks; kk < kTR; kk += 16 * KS) {            // Eq. 2.5: 16 rows of the tile per instruction
#pragma unroll
            for (int t = 0; t < NBLK; ++t) {
                const int q = wq + 4 * t, bi = q / TNB, bj = q % TNB;
                acc_w[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_strided(Ps + (kk + 8 * lh) * SP + 32 * bi + l32, SP),
                                                                   frag_strided(Qs + (kk + 8 * lh) * SQ + 32 * bj + l32, SQ),
                                                                   acc_w[t], 0, 0, 0);
            }
        }
        __syncthreads();
        commit();
        if (dOut) {
#pragma unroll
            for (int c = 0; c < NCB; ++c) {
                const int gc = 16 * c + l16;
                if (gc < Mp) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int64_t gr = r0 + 16 * w + 4 * lq + r;
                        if (gr < r_end) dOut[gr * ldo + gc] = f32_to_bf16(acc_o[c][r]);
                    }
                }
            }
        }
        __syncthreads();
    }

    float* out = part + ((int64_t)blockIdx.x * KS + ks) * Mp * N;
#pragma unroll
    for (int t = 0; t < NBLK; ++t) {
        const int q = wq + 4 * t, bi = q / TNB, bj = q % TNB;
        const int gn = 32 * bj + l32;
        if (gn >= N) continue;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int gm = 32 * bi + 8 * (r / 4) + 4 * lh + (r % 4);
            if (gm < Mp) out[(int64_t)gm * N + gn] = acc_w[t][r];
        }
    }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

template <typename Kern>
plx_status set_lds(plx_ctx* ctx, Kern kern, size_t lds) {
    if (lds > 48 * 1024)
        PLX_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    return PLX_OK;
}

template <int TMB, int TNB, bool MASK>
plx_status run_bwd(plx_ctx* ctx, int64_t R, int Mp, int N, const bf16_t* P, int64_t ldp, const bf16_t* Q, int64_t ldq,
                   const bf16_t* Zm, int64_t ldz, const float* W, int64_t ldw, bf16_t* dOut, int64_t ldo, float* part,
                   int64_t rpc, int64_t chunks) {
    constexpr int MP = 32 * TMB, NP = 32 * TNB;
    const size_t lds = sizeof(bf16_t) * (kTR * (NP + 8) + kTR * (MP + 8) + MP * (NP + 8));
    const int vec_p = aligned16(P) && ldp % 8 == 0;
    const int vec_q = aligned16(Q) && ldq % 8 == 0 && (!Zm || (aligned16(Zm) && ldz % 8 == 0));
    auto kern = k_bwd_dense_bf16<TMB, TNB, MASK>;
    PLX_TRY(set_lds(ctx, kern, lds));
    kern<<<dim3((unsigned)chunks), 256, lds, ctx->stream>>>(R, Mp, N, P, ldp, Q, ldq, Zm, ldz, W, ldw, dOut, ldo, part, rpc,
                                                           vec_p, vec_q);
    PLX_HIP(ctx, hipGetLastError());
    return PLX_OK;
}

}  // namespace

plx_status launch_gemm_small_bf16(plx_ctx* ctx, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                                  const float* W, int64_t ldw, void* C, int64_t ldc, void* Fact, int64_t ldf) {
    if (K > 128 || N > 128 || K <= 0) return fail(ctx, PLX_ERR_UNSUPPORTED, "bf16 dense products are built for widths up to 128");
    const int tkb = K <= 32 ? 1 : (K <= 64 ? 2 : 4), tnb = N <= 32 ? 1 : (N <= 64 ? 2 : 4);
    const int rb = tnb == 1 ? 4 : 2, rows = 32 * rb;
    const size_t lds = sizeof(bf16_t) * (2 * rows * (32 * tkb + 8) + 32 * tnb * (32 * tkb + 8));
    const int per_cu = (int)std::max<size_t>(1, std::min<size_t>(8, (150 * 1024) / lds));
    const int64_t blocks = std::min<int64_t>(ceil_div(M, rows), (int64_t)ctx->n_cu * per_cu);
    const int vec_a = aligned16(A) && lda % 8 == 0;
    char label[64];
    snprintf(label, sizeof label, "gemm_nn<bf16>[M%lld,N%lld,K%lld]", (long long)M, (long long)N, (long long)K);
    KernelTimer kt(ctx, label);
#define PLX_SMALL(TK, TN, RBV)                                                                                  \
    do {                                                                                                        \
        auto kern = k_gemm_small_bf16<TK, TN, RBV>;                                                             \
        PLX_TRY(set_lds(ctx, kern, lds));                                                                       \
        kern<<<dim3((unsigned)blocks), 256, lds, ctx->stream>>>(M, (int)N, (int)K, (const bf16_t*)A, lda, W, ldw, \
                                                               (bf16_t*)C, ldc, (bf16_t*)Fact, ldf, vec_a);     \
    } while (0)
    switch (tkb * 10 + tnb) {
        case 11: PLX_SMALL(1, 1, 4); break;
        case 12: PLX_SMALL(1, 2, 2); break;
        case 14: PLX_SMALL(1, 4, 2); break;
        case 21: PLX_SMALL(2, 1, 4); break;
        case 22: PLX_SMALL(2, 2, 2); break;
        case 24: PLX_SMALL(2, 4, 2); break;
        case 41: PLX_SMALL(4, 1, 4); break;
        case 42: PLX_SMALL(4, 2, 2); break;
        default: PLX_SMALL(4, 4, 2); break;
    }
#undef PLX_SMALL
    PLX_HIP(ctx, hipGetLastError());
    return PLX_OK;
}

plx_status launch_bwd_dense_bf16(plx_ctx* ctx, int64_t R, int64_t Mp, int64_t N, const void* P, int64_t ldp, const void* Q,
                                 int64_t ldq, const void* Zm, int64_t ldz, const float* W, int64_t ldw, void* dOut,
                                 int64_t ldo, float* dW, int64_t lddw, void* ws, size_t ws_bytes) {
    if (Mp > 128 || N > 128) return fail(ctx, PLX_ERR_UNSUPPORTED, "bf16 dense products are built for widths up to 128");
    if (ws_bytes < gemm_tn_workspace(R, Mp, N)) return fail(ctx, PLX_ERR_SHAPE, "workspace too small");
    const int64_t rpc = tn_rows_per_chunk(R, Mp, N);
    const int64_t chunks = std::max<int64_t>(1, ceil_div(R, rpc));
    float* part = static_cast<float*>(ws);
    const int tmb = Mp <= 32 ? 1 : (Mp <= 64 ? 2 : 4), tnb = N <= 32 ? 1 : (N <= 64 ? 2 : 4);
    char label[64];
    snprintf(label, sizeof label, "bwd_dense<bf16>[R%lld,M%lld,N%lld]", (long long)R, (long long)Mp, (long long)N);
    plx_status st;
    {
        KernelTimer kt(ctx, label);
#define PLX_BD(TM, TN)                                                                                                  \
    st = Zm ? run_bwd<TM, TN, true>(ctx, R, (int)Mp, (int)N, (const bf16_t*)P, ldp, (const bf16_t*)Q, ldq,              \
                                    (const bf16_t*)Zm, ldz, W, ldw, (bf16_t*)dOut, ldo, part, rpc, chunks)              \
            : run_bwd<TM, TN, false>(ctx, R, (int)Mp, (int)N, (const bf16_t*)P, ldp, (const bf16_t*)Q, ldq, nullptr, 0, \
                                     W, ldw, (bf16_t*)dOut, ldo, part, rpc, chunks)
        switch (tmb * 10 + tnb) {
            case 11: PLX_BD(1, 1); break;
            case 12: PLX_BD(1, 2); break;
            case 14: PLX_BD(1, 4); break;
            case 21: PLX_BD(2, 1); break;
            case 22: PLX_BD(2, 2); break;
            case 24: PLX_BD(2, 4); break;
            case 41: PLX_BD(4, 1); break;
            case 42: PLX_BD(4, 2); break;
            default: PLX_BD(4, 4); break;
        }
#undef PLX_BD
    }
    PLX_TRY(st);
    return reduce_partials(ctx, part, chunks * tn_kslices(Mp, N), Mp, N, dW, lddw);
}

}  // namespace plx
