// Dense products of a GCN layer with bf16 storage and fp32 accumulation (Eq. 2.2, 2.3 forward;
// Eq. 2.4, 2.5, 2.6 fused backward), for widths up to 128.  Activations and gradients are bf16 in
// HBM, the weight matrix is fp32 in HBM and rounded to bf16 (nearest even) when a wavefront loads
// its share into registers, products are exact in fp32 and accumulated in fp32 by
// v_mfma_f32_32x32x16_bf16 / v_mfma_f32_16x16x32_bf16.  At these widths the matrix work is a few
// percent of the time: the kernels are streaming kernels bound by HBM, organised like their fp32
// counterparts (weights in registers, LDS holds only row tiles, next tile prefetched into
// registers during the MFMAs, unconditional prefetch).
//
// Operand convention of both instructions: lane l supplies 8 consecutive k-values of row/column
// (l % 32 or l % 16), the k-slab chosen by l / 32 (or l / 16).  Both operands are fed with the
// same slab mapping, so the contraction is over all k whatever the hardware's numbering.
// Accumulator layouts equal those of the fp32 instructions of the same tile shape.
//
// Where the contraction runs over the ROWS of a row-major LDS tile (dW = P^T Q'), an operand is a
// column of the tile.  It is fetched with the LDS transpose read of gfx950 (ds_read_b64_tr_b16):
// inside each group of 16 lanes, lane L passes the address of 4 consecutive elements of row
// L / 4, columns 4*(L % 4).., and receives rows 0..3 of column L of that 4 x 16 block.
//
// Results leave through a small per-wavefront LDS staging area so that every lane stores 16
// bytes (8 bf16) with one non-temporal store instead of eight 2-byte stores.
#include "plx_internal.h"
#include "buffer_addr.h"
#include "bf16_frag.h"

#include <algorithm>

namespace plx {
namespace {

// guarded load of 8 consecutive bf16 of a global row (zero beyond ncols / the last row).  With
// vec (16-byte aligned base and leading dimension) a chunk that straddles ncols still lies inside
// the row's pitch: it is loaded whole and the surplus elements are zeroed -- except on the very
// last row of the matrix, where the bytes behind the last column need not exist.
__device__ __forceinline__ uint4 load8(const bf16_t* __restrict__ src, int64_t ld, int64_t gr, int64_t r_end,
                                       int64_t r_total, int gc, int ncols, bool vec) {
    Frag f;
    f.u = make_uint4(0, 0, 0, 0);
    if (gr < r_end && gc < ncols) {
        const bf16_t* p = src + gr * ld + gc;
        if (vec && (gc + 7 < ncols || gr + 1 < r_total)) {
            f.u = *reinterpret_cast<const uint4*>(p);
            if (gc + 7 >= ncols) {
#pragma unroll
                for (int i = 1; i < 8; ++i)
                    if (gc + i >= ncols) f.e[i] = 0;
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (gc + i < ncols) f.e[i] = p[i];
        }
    }
    return f.u;
}

// Buffer-addressed form of the same load (16-byte aligned rows): `off` is the piece's byte offset inside
// the tile, computed once per kernel (pieces wholly past ncols carry an offset the descriptor never
// reaches), and the descriptor ends with column ncols of the last valid row, so nothing is tested per
// lane.  Only a piece that straddles ncols (ncols % 8 != 0) needs its surplus elements zeroed.
__device__ __forceinline__ uint32_t piece_offset(int f, int pieces, int per_row, int64_t ld, int ncols) {
    const int r = f / per_row, q = f % per_row;
    return (f < pieces && 8 * q < ncols) ? (uint32_t)(((uint32_t)r * (uint32_t)ld + 8u * q) * 2u) : kOutOfRange;
}
__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_buffer(const bf16_t* base, int64_t ld, int64_t row0, int64_t r_end,
                                                              int tile_rows, int ncols) {
    const int64_t left = r_end - row0;
    const int64_t rows = left < tile_rows ? left : tile_rows;
    // the range check works on whole 32-bit words: with an odd ncols the word that holds the last column
    // must count as inside (its other half is padding of the same 16-byte aligned row)
    return buffer_of(base + row0 * ld, rows > 0 ? (uint32_t)((((rows - 1) * ld + ncols) * 2 + 3) & ~int64_t(3)) : 0u);
}
__device__ __forceinline__ uint4 load8_buf(__amdgpu_buffer_rsrc_t rs, uint32_t off, int gc, int ncols) {
    Frag f;
    f.u = __builtin_bit_cast(uint4, buffer_load4(rs, off));
    if (ncols & 7) {                                   // uniform
#pragma unroll
        for (int i = 1; i < 8; ++i)
            if (gc + i >= ncols) f.e[i] = 0;
    }
    return f.u;
}

// Buffer-addressed write-out of a staged block (destination rows 16-byte aligned): the lane's pieces
// sit at byte offsets `off[k]` inside the block (computed once per kernel; pieces not wholly inside
// the ncols columns carry an unreachable offset), the descriptor ends with the last valid row.
// A piece that straddles ncols (ncols % 8 != 0) is written element by element.
template <int COLS, int NPC>
__device__ __forceinline__ void stage_store_buf(const bf16_t* stage, int nrows, bf16_t* __restrict__ dst, int64_t ld,
                                                int64_t row0, int64_t r_end, int col0, int ncols, const uint32_t (&off)[NPC],
                                                int lane) {
    constexpr int PITCH = COLS + 8, CH = COLS / 8;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const __amdgpu_buffer_rsrc_t rs = tile_buffer(dst, ld, row0, r_end, nrows, ncols);
#pragma unroll
    for (int k = 0; k < NPC; ++k) {
        const int i = lane + 64 * k, r = i / CH, c = 8 * (i % CH);
        Frag f;
        f.u = *reinterpret_cast<const uint4*>(stage + (r % nrows) * PITCH + c);
        __builtin_amdgcn_raw_buffer_store_b128(f.x, rs, (int)off[k], 0, 2);
        if ((ncols & 7) && i < nrows * CH) {            // first condition uniform
            const int gc = col0 + c;
            const int64_t gr = row0 + r;
            if (gr < r_end && gc < ncols && gc + 7 >= ncols) {
                bf16_t* p = dst + gr * ld + gc;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (gc + e < ncols) p[e] = f.e[e];
            }
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}
// byte offset of piece i of a staged nrows x COLS block whose first column is col0 (see stage_store_buf)
template <int COLS>
__device__ __forceinline__ uint32_t stage_offset(int i, int nrows, int64_t ld, int col0, int ncols) {
    constexpr int CH = COLS / 8;
    const int r = i / CH, gc = col0 + 8 * (i % CH);
    return (i < nrows * CH && gc + 7 < ncols) ? (uint32_t)(((uint32_t)r * (uint32_t)ld + gc) * 2u) : kOutOfRange;
}

// One wavefront writes a ROWS16*16 x COLS block of results: the values go through the
// wavefront's own staging area (row-major, pitch COLS + 8) and leave as 16-byte non-temporal
// stores when the destination allows it (vec), else as single elements.  LDS operations of one
// wavefront execute in order, so no barrier is needed between the two phases; the fences keep
// the compiler from reordering them.
template <int COLS>
__device__ __forceinline__ void stage_store(bf16_t* stage, int nrows, bf16_t* __restrict__ dst, int64_t ld, int64_t row0,
                                            int64_t r_end, int col0, int ncols, bool vec, int lane) {
    constexpr int PITCH = COLS + 8, CH = COLS / 8;            // 16-byte chunks per row
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (int i = lane; i < nrows * CH; i += 64) {
        const int r = i / CH, c = 8 * (i % CH);
        const int64_t gr = row0 + r;
        const int gc = col0 + c;
        if (gr >= r_end || gc >= ncols) continue;
        Frag f;
        f.u = *reinterpret_cast<const uint4*>(stage + r * PITCH + c);
        bf16_t* p = dst + gr * ld + gc;
        if (vec && gc + 7 < ncols) {
            __builtin_nontemporal_store(f.x, reinterpret_cast<u32x4*>(p));
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (gc + e < ncols) p[e] = f.e[e];
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// ---- forward: C[M x N] = A[M x K] W[K x N] (+ ReLU copy), K, N <= 128 --------------------------------
// Block q = w + 4t of the RB x TNB grid of 32x32 blocks belongs to wavefront w; 4 % TNB == 0, so a
// wavefront always works on column block w % TNB and keeps that slice of W in registers.
template <int TKB, int TNB, int RB>
__global__ __launch_bounds__(256) void k_gemm_small_bf16(int64_t M, int N, int K, const bf16_t* __restrict__ A,
                                                         int64_t lda, const float* __restrict__ W, int64_t ldw,
                                                         bf16_t* __restrict__ C, int64_t ldc, bf16_t* __restrict__ F,
                                                         int64_t ldf, uint32_t* __restrict__ bits, int64_t ldbits, int vec_a,
                                                         int vec_c, int vec_f, int bits_vec) {
    constexpr int KP = 32 * TKB, ROWS = 32 * RB;
    constexpr int NBLK = RB * TNB / 4, NKS = KP / 16;
    constexpr int NLD = (ROWS * KP / 8 + 255) / 256;       // 16-byte pieces per thread per tile
    constexpr int SA = KP + 8;                              // LDS row pitch in elements (16-byte multiple)
    static_assert((RB * TNB) % 4 == 0 && 4 % TNB == 0, "tile must split evenly over 4 wavefronts");
    extern __shared__ __align__(16) unsigned char smem_raw[];
    bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
    auto a_buf = [&](int b) { return smem + b * ROWS * SA; };
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5;
    const int bj = w % TNB;
    bf16_t* stage = smem + 2 * ROWS * SA + w * 32 * 40;    // per wavefront: 32 rows x (32 + 8)
    // sign bits of a tile (only when bits != NULL): two buffers [word][row]; the wavefronts drop their
    // ballots here and the words leave one tile later as one store per row
    uint32_t* sb = reinterpret_cast<uint32_t*>(smem + 2 * ROWS * SA + 4 * 32 * 40);

    bf16x8 breg[NKS];                                       // breg[s] = W[16s + 8*lh .. +7][32*bj + l32]
    {
        const int n = 32 * bj + l32;
#pragma unroll
        for (int s2 = 0; s2 < NKS; ++s2) {
            Frag f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int kk = 16 * s2 + 8 * lh + e;
                f.e[e] = (kk < K && n < N) ? f32_to_bf16(W[(int64_t)kk * ldw + n]) : (bf16_t)0;
            }
            breg[s2] = f.v;
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);    // weights landed before the row loop (vmcnt(0))

    const int64_t n_tiles = (M + ROWS - 1) / ROWS;
    uint4 reg[NLD];
    uint32_t toff[NLD];                                     // vec_a: byte offsets of the thread's pieces inside a tile
#pragma unroll
    for (int i = 0; i < NLD; ++i) toff[i] = piece_offset(tid + 256 * i, ROWS * KP / 8, KP / 8, lda, K);
    auto fetch = [&](int64_t tile) {
        if (vec_a) {                                        // uniform
            const __amdgpu_buffer_rsrc_t ra = tile_buffer(A, lda, tile * ROWS, M, ROWS, K);
#pragma unroll
            for (int i = 0; i < NLD; ++i) reg[i] = load8_buf(ra, toff[i], 8 * ((tid + 256 * i) % (KP / 8)), K);
            return;
        }
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int f = tid + 256 * i, r = f / (KP / 8), q = f % (KP / 8);
            reg[i] = (f < ROWS * KP / 8) ? load8(A, lda, tile * ROWS + r, M, M, 8 * q, K, false) : make_uint4(0, 0, 0, 0);
        }
    };
    // write-out: piece k of a wavefront's staged 32 x 32 block (see stage_store_buf)
    uint32_t coff[2], foff[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        coff[k] = stage_offset<32>(lane + 64 * k, 32, ldc, 32 * bj, N);
        foff[k] = stage_offset<32>(lane + 64 * k, 32, ldf, 32 * bj, N);
    }
    auto commit = [&](bf16_t* As) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int f = tid + 256 * i, r = f / (KP / 8), q = f % (KP / 8);
            if (f < ROWS * KP / 8) *reinterpret_cast<uint4*>(As + r * SA + 8 * q) = reg[i];
        }
    };

    const int nw = (N + 31) >> 5;
    auto flush_bits = [&](int buf, int64_t t) {             // words of tile t, written by the pass before
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
    if (tile < n_tiles) { fetch(tile); commit(a_buf(0)); }
    __syncthreads();
    const int k_end = (K + 15) & ~15;
    for (; tile < n_tiles; tile += gridDim.x) {
        // unconditional prefetch (the last pass re-reads its own tile): straight-line code keeps the
        // only wait for loads right before the LDS write
        fetch(tile + gridDim.x < n_tiles ? tile + gridDim.x : tile);
        if (bits && prev >= 0) flush_bits(cur ^ 1, prev);
        prev = tile;
        const bf16_t* As = a_buf(cur);
        floatx16 acc[NBLK];
#pragma unroll
        for (int t = 0; t < NBLK; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
#pragma unroll
        for (int s2 = 0; s2 < NKS; ++s2) {
            if (16 * s2 >= k_end) break;                    // uniform
#pragma unroll
            for (int t = 0; t < NBLK; ++t) {
                const int bi = (w + 4 * t) / TNB;
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_contig(As + (32 * bi + l32) * SA + 16 * s2 + 8 * lh),
                                                                 breg[s2], acc[t], 0, 0, 0);
            }
        }
        commit(a_buf(cur ^ 1));
        const int64_t m0 = tile * ROWS;
#pragma unroll
        for (int t = 0; t < NBLK; ++t) {
            const int bi = (w + 4 * t) / TNB;
            if (32 * bj >= N) continue;
            if (C) {                                        // plain result
#pragma unroll
                for (int r = 0; r < 16; ++r) stage[(8 * (r / 4) + 4 * lh + (r % 4)) * 40 + l32] = f32_to_bf16(acc[t][r]);
                if (vec_c) stage_store_buf<32, 2>(stage, 32, C, ldc, m0 + 32 * bi, M, 32 * bj, N, coff, lane);
                else stage_store<32>(stage, 32, C, ldc, m0 + 32 * bi, M, 32 * bj, N, false, lane);
            }
            if (F) {                                        // its ReLU (Eq. 2.3), and the sign of the rounded value
                bf16_t h[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    h[r] = f32_to_bf16(relu0(acc[t][r]));
                    stage[(8 * (r / 4) + 4 * lh + (r % 4)) * 40 + l32] = h[r];
                }
                if (vec_f) stage_store_buf<32, 2>(stage, 32, F, ldf, m0 + 32 * bi, M, 32 * bj, N, foff, lane);
                else stage_store<32>(stage, 32, F, ldf, m0 + 32 * bi, M, 32 * bj, N, false, lane);
                if (bits) {    // one ballot = 32 columns of two rows (lanes 0-31, lanes 32-63); max(v, 0) rounds to 0 or to a positive value
                    // the ballots are wave-uniform: lane 0 stores both halves, 8 consecutive rows per step
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        uint32_t lo[4], hi[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const unsigned long long b = __ballot((h[4 * g + j] & 0x7fffu) != 0);
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
        }
        __syncthreads();
        cur ^= 1;
    }
    if (bits && prev >= 0) flush_bits(cur ^ 1, prev);       // the last pass ended with a barrier
}

// ---- backward: dOut = (Q*[Zm>0]) W^T, dW partial = P^T (Q*[Zm>0]) ---------------------------------------
#ifndef PLX_BF16_TR
#define PLX_BF16_TR 32
#endif
constexpr int kTR = PLX_BF16_TR;      // rows per tile

template <int TMB, int TNB, int MASK>   // MASK: 0 none, 1 Zm holds values, 2 Zm holds sign bits (ldz in words)
__global__ __launch_bounds__(256) void k_bwd_dense_bf16(int64_t R, int Mp, int N, const bf16_t* __restrict__ P,
                                                        int64_t ldp, const bf16_t* __restrict__ Q, int64_t ldq,
                                                        const bf16_t* __restrict__ Zm, int64_t ldz,
                                                        const float* __restrict__ W, int64_t ldw,
                                                        bf16_t* __restrict__ dOut, int64_t ldo, float* __restrict__ part,
                                                        int64_t rows_per_chunk, int vec_p, int vec_q, int vec_o) {
    constexpr int MP = 32 * TMB, NP = 32 * TNB, SQ = NP + 8, SP = MP + 8;
    constexpr int NB = TMB * TNB, KS = NB >= 4 ? 1 : 4 / NB, NBLK = NB >= 4 ? NB / 4 : 1;
    // dOut tile = (kTR/16) x NCB blocks of 16x16; a wavefront owns NCW column blocks (their W rows
    // live in its registers) of NRW row blocks: Mp >= 64: column blocks w*NCW.., all row blocks;
    // Mp <= 32: column block w/2 of row blocks w%2, w%2 + 2, ...
    constexpr int NCB = MP / 16, NCW = NCB >= 4 ? NCB / 4 : 1, NRW = NCB >= 4 ? kTR / 16 : kTR / 32, NKS = NP / 32;
    constexpr int NQ = (kTR * NP / 8 + 255) / 256, NPR = (kTR * MP / 8 + 255) / 256;   // 16-byte pieces per thread
    constexpr int SO = 16 * NCW + 8;                                           // staging pitch
    extern __shared__ __align__(16) unsigned char smem_raw[];
    bf16_t* Qs = reinterpret_cast<bf16_t*>(smem_raw);
    bf16_t* Ps = Qs + kTR * SQ;
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5, l16 = lane & 15, lq = lane >> 4;
    const int wq = NB >= 4 ? w : w % NB, ks = NB >= 4 ? 0 : w / NB;
    const int cb0 = NCB >= 4 ? w * NCW : (w >> 1), rb0 = NCB >= 4 ? 0 : (w & 1), rbs = NCB >= 4 ? 1 : 2;
    bf16_t* stage = Ps + kTR * SP + w * 16 * SO;            // per wavefront: 16 rows x (16*NCW + 8)
    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_chunk;
    const int64_t r_end = (r_begin + rows_per_chunk < R) ? r_begin + rows_per_chunk : R;

    bf16x8 wreg[NCW][NKS];                                  // wreg[c][s] = W[16*(cb0+c) + l16][32s + 8*lq .. +7]
#pragma unroll
    for (int c = 0; c < NCW; ++c) {
        const int i = 16 * (cb0 + c) + l16;
#pragma unroll
        for (int s2 = 0; s2 < NKS; ++s2) {
            Frag f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int n = 32 * s2 + 8 * lq + e;
                f.e[e] = (W && dOut && i < Mp && n < N) ? f32_to_bf16(W[(int64_t)i * ldw + n]) : (bf16_t)0;
            }
            wreg[c][s2] = f.v;
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);    // weights landed before the row loop (vmcnt(0))

    floatx16 acc_w[NBLK];
#pragma unroll
    for (int t = 0; t < NBLK; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_w[t][r] = 0.f;

    uint4 rq[NQ], rz[NQ], rp[NPR];
    // MASK == 2: piece i of thread tid (8 columns) lies in word tid / 4 + 64 i of the tile's 32 * NP / 32
    // words; lane l < 16 * NQ loads word 16 * wavefront + l % 16 + 64 * (l / 16), and at commit time
    // piece i takes its word from lane l / 4 + 16 i and its byte at bit 8 * (tid % 4)
    static_assert(MASK != 2 || kTR == 32, "word numbering assumes 32-row tiles");
    uint32_t zb = 0;
    const uint32_t* Zbits = reinterpret_cast<const uint32_t*>(Zm);
    // byte offsets, inside a tile, of the thread's pieces (vec_q / vec_p) and of its sign word
    uint32_t oq[NQ], oz[NQ], op[NPR], ob = kOutOfRange;
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
        oq[i] = piece_offset(tid + 256 * i, kTR * NP / 8, NP / 8, ldq, N);
        oz[i] = MASK == 1 ? piece_offset(tid + 256 * i, kTR * NP / 8, NP / 8, ldz, N) : 0u;
    }
#pragma unroll
    for (int i = 0; i < NPR; ++i) op[i] = piece_offset(tid + 256 * i, kTR * MP / 8, MP / 8, ldp, Mp);
    if (MASK == 2) {
        constexpr int WPR = NP / 32;
        const int wi = 16 * w + (lane & 15) + 64 * (lane >> 4), cw = wi % WPR;
        if (lane < 16 * NQ && wi < 32 * WPR && 32 * cw < N) ob = (uint32_t)(((uint32_t)(wi / WPR) * (uint32_t)ldz + cw) * 4u);
    }
    auto fetch = [&](int64_t r0) {
        if (vec_q) {                                                  // uniform
            const __amdgpu_buffer_rsrc_t bq = tile_buffer(Q, ldq, r0, r_end, kTR, N);
#pragma unroll
            for (int i = 0; i < NQ; ++i) rq[i] = load8_buf(bq, oq[i], 8 * ((tid + 256 * i) % (NP / 8)), N);
            if (MASK == 1) {
                const __amdgpu_buffer_rsrc_t bz = tile_buffer(Zm, ldz, r0, r_end, kTR, N);
#pragma unroll
                for (int i = 0; i < NQ; ++i) rz[i] = load8_buf(bz, oz[i], 8 * ((tid + 256 * i) % (NP / 8)), N);
            }
        } else {
#pragma unroll
            for (int i = 0; i < NQ; ++i) {
                const int f = tid + 256 * i, r = f / (NP / 8), q = f % (NP / 8);
                const bool in = f < kTR * NP / 8;
                rq[i] = in ? load8(Q, ldq, r0 + r, r_end, R, 8 * q, N, false) : make_uint4(0, 0, 0, 0);
                if (MASK == 1) rz[i] = in ? load8(Zm, ldz, r0 + r, r_end, R, 8 * q, N, false) : make_uint4(0, 0, 0, 0);
            }
        }
        if (vec_p) {
            const __amdgpu_buffer_rsrc_t bp = tile_buffer(P, ldp, r0, r_end, kTR, Mp);
#pragma unroll
            for (int i = 0; i < NPR; ++i) rp[i] = load8_buf(bp, op[i], 8 * ((tid + 256 * i) % (MP / 8)), Mp);
        } else {
#pragma unroll
            for (int i = 0; i < NPR; ++i) {
                const int f = tid + 256 * i, r = f / (MP / 8), q = f % (MP / 8);
                rp[i] = (f < kTR * MP / 8) ? load8(P, ldp, r0 + r, r_end, R, 8 * q, Mp, false) : make_uint4(0, 0, 0, 0);
            }
        }
        if (MASK == 2) {                                              // descriptor in words: rows past the chunk read 0
            const int64_t left = r_end - r0;
            const int64_t rows = left < kTR ? left : kTR;
            zb = buffer_load1(buffer_of(Zbits + r0 * ldz, rows > 0 ? (uint32_t)(((rows - 1) * ldz + (N + 31) / 32) * 4) : 0u), ob);
        }
    };
    uint32_t ooff[1];                                                 // write-out of a wavefront's staged 16 x 16*NCW block
    ooff[0] = stage_offset<16 * NCW>(lane, 16, ldo, 16 * cb0, Mp);
    static_assert(16 * (16 * NCW / 8) <= 64, "one piece per lane");
    auto commit = [&]() {
#pragma unroll
        for (int i = 0; i < NQ; ++i) {
            const int f = tid + 256 * i, r = f / (NP / 8), q = f % (NP / 8);
            Frag v;
            v.u = rq[i];
            if (MASK == 1) {                                         // Eq. 2.4
                Frag z;
                z.u = rz[i];
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (!bf16_positive(z.e[e])) v.e[e] = 0;
            } else if (MASK == 2) {
                // two elements per word: bits e and e + 1 of the byte, each spread over its half-word
                const int b = (int)__shfl(zb, (lane >> 2) + 16 * i);
                const unsigned s0 = 8 * (tid & 3);
                u32x4 m;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    m[e] = ((unsigned)__builtin_amdgcn_sbfe(b, s0 + 2 * e, 1) & 0xffffu) | ((unsigned)__builtin_amdgcn_sbfe(b, s0 + 2 * e + 1, 1) & 0xffff0000u);
                v.x &= m;
            }
            if (f < kTR * NP / 8) *reinterpret_cast<uint4*>(Qs + r * SQ + 8 * q) = v.u;
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
    const int n_end = (N + 31) & ~31;
    for (int64_t r0 = r_begin; r0 < r_end; r0 += kTR) {
        fetch(r0 + kTR < r_end ? r0 + kTR : r0);      // unconditional, as in the forward kernel

        floatx4 acc_o[NRW][NCW];
        if (dOut) {                                                  // Eq. 2.6
#pragma unroll
            for (int rr = 0; rr < NRW; ++rr)
#pragma unroll
                for (int c = 0; c < NCW; ++c) acc_o[rr][c] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s2 = 0; s2 < NKS; ++s2) {
                if (32 * s2 >= n_end) break;                          // uniform
#pragma unroll
                for (int rr = 0; rr < NRW; ++rr) {
                    const bf16x8 a = frag_contig(Qs + (16 * (rb0 + rbs * rr) + l16) * SQ + 32 * s2 + 8 * lq);
#pragma unroll
                    for (int c = 0; c < NCW; ++c)
                        acc_o[rr][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, wreg[c][s2], acc_o[rr][c], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int kk = 16 * ks; kk < kTR; kk += 16 * KS) {            // Eq. 2.5: 16 rows of the tile per instruction
#pragma unroll
            for (int t = 0; t < NBLK; ++t) {
                const int q = wq + 4 * t, bi = q / TNB, bj = q % TNB;
                acc_w[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_column(Ps, SP, kk, 32 * bi, lane),
                                                                   frag_column(Qs, SQ, kk, 32 * bj, lane), acc_w[t], 0, 0, 0);
            }
        }
        __syncthreads();
        commit();
        if (dOut) {
#pragma unroll
            for (int rr = 0; rr < NRW; ++rr) {
#pragma unroll
                for (int c = 0; c < NCW; ++c)
#pragma unroll
                    for (int r = 0; r < 4; ++r) stage[(4 * lq + r) * SO + 16 * c + l16] = f32_to_bf16(acc_o[rr][c][r]);
                if (vec_o) stage_store_buf<16 * NCW, 1>(stage, 16, dOut, ldo, r0 + 16 * (rb0 + rbs * rr), r_end, 16 * cb0, Mp, ooff, lane);
                else stage_store<16 * NCW>(stage, 16, dOut, ldo, r0 + 16 * (rb0 + rbs * rr), r_end, 16 * cb0, Mp, false, lane);
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

template <int TMB, int TNB, int MASK>
plx_status run_bwd(plx_ctx* ctx, int64_t R, int Mp, int N, const bf16_t* P, int64_t ldp, const bf16_t* Q, int64_t ldq,
                   const bf16_t* Zm, int64_t ldz, const float* W, int64_t ldw, bf16_t* dOut, int64_t ldo, float* part,
                   int64_t rpc, int64_t chunks) {
    constexpr int MP = 32 * TMB, NP = 32 * TNB;
    constexpr int NCW = MP / 16 >= 4 ? MP / 64 : 1;
    const size_t lds = sizeof(bf16_t) * (kTR * (NP + 8) + kTR * (MP + 8) + 4 * 16 * (16 * NCW + 8));
    const int vec_p = aligned16(P) && ldp % 8 == 0;
    const int vec_q = aligned16(Q) && ldq % 8 == 0 && (MASK != 1 || (aligned16(Zm) && ldz % 8 == 0));
    const int vec_o = aligned16(dOut) && ldo % 8 == 0;
    auto kern = k_bwd_dense_bf16<TMB, TNB, MASK>;
    PLX_TRY(set_lds(ctx, kern, lds));
    kern<<<dim3((unsigned)chunks), 256, lds, ctx->stream>>>(R, Mp, N, P, ldp, Q, ldq, Zm, ldz, W, ldw, dOut, ldo, part, rpc,
                                                           vec_p, vec_q, vec_o);
    PLX_HIP(ctx, hipGetLastError());
    return PLX_OK;
}

}  // namespace

#ifndef PLX_BF16_FWD_CAP
#define PLX_BF16_FWD_CAP 3            // resident workgroups per CU of the forward kernel (0: as many as fit); measured: 3 is
                                      // 5 % faster than 4+ at 32 -> 128 and 19 % faster at 64 -> 128, equal elsewhere; 2 is slower
#endif
plx_status launch_gemm_small_bf16(plx_ctx* ctx, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                                  const float* W, int64_t ldw, void* C, int64_t ldc, void* Fact, int64_t ldf,
                                  uint32_t* bits, int64_t ldbits) {
    if (K > 128 || N > 128 || K <= 0) return fail(ctx, PLX_ERR_UNSUPPORTED, "bf16 dense products are built for widths up to 128");
    // a tile (up to 128 rows) is addressed with 31-bit byte offsets
    if (lda >= (int64_t(1) << 23) || (C && ldc >= (int64_t(1) << 23)) || (Fact && ldf >= (int64_t(1) << 23)))
        return fail(ctx, PLX_ERR_UNSUPPORTED, "leading dimensions of 2^23 elements or more are not supported by the bf16 dense kernels");
    const int tkb = K <= 32 ? 1 : (K <= 64 ? 2 : 4), tnb = N <= 32 ? 1 : (N <= 64 ? 2 : 4);
    const int rb = tnb == 1 ? 4 : 2, rows = 32 * rb;
    const size_t lds = sizeof(bf16_t) * (2 * rows * (32 * tkb + 8) + 4 * 32 * 40) + (bits ? 2 * 4 * rows * 4 : 0);
    const int nw = (int)ceil_div(N, 32);
    const uintptr_t bp = reinterpret_cast<uintptr_t>(bits);
    const int bits_vec = (nw == 4 && ldbits % 4 == 0 && bp % 16 == 0) ? 4 : ((nw == 2 && ldbits % 2 == 0 && bp % 8 == 0) ? 2 : 1);
    const int vec_a = aligned16(A) && lda % 8 == 0;
    const int vec_c = C && aligned16(C) && ldc % 8 == 0, vec_f = Fact && aligned16(Fact) && ldf % 8 == 0;
    char label[64];
    snprintf(label, sizeof label, "gemm_nn<bf16>[M%lld,N%lld,K%lld]", (long long)M, (long long)N, (long long)K);
    KernelTimer kt(ctx, label);
#define PLX_SMALL(TK, TN, RBV)                                                                                  \
    do {                                                                                                        \
        auto kern = k_gemm_small_bf16<TK, TN, RBV>;                                                             \
        PLX_TRY(set_lds(ctx, kern, lds));                                                                       \
        int per_cu = 0;                                                                                         \
        PLX_HIP(ctx, hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, 256, lds));                    \
        if (PLX_BF16_FWD_CAP > 0) per_cu = std::min(per_cu, PLX_BF16_FWD_CAP);                                  \
        const int64_t blocks = std::min<int64_t>(ceil_div(M, rows), (int64_t)ctx->n_cu * std::max(1, per_cu));  \
        kern<<<dim3((unsigned)blocks), 256, lds, ctx->stream>>>(M, (int)N, (int)K, (const bf16_t*)A, lda, W, ldw, \
                                                               (bf16_t*)C, ldc, (bf16_t*)Fact, ldf, bits, ldbits, \
                                                               vec_a, vec_c, vec_f, bits_vec);                   \
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
                                 int64_t ldo, float* dW, int64_t lddw, void* ws, size_t ws_bytes, bool mask_bits) {
    if (Mp > 128 || N > 128) return fail(ctx, PLX_ERR_UNSUPPORTED, "bf16 dense products are built for widths up to 128");
    if (ws_bytes < gemm_tn_workspace(R, Mp, N)) return fail(ctx, PLX_ERR_SHAPE, "workspace too small");
    const int64_t rpc = tn_rows_per_chunk(R, Mp, N);
    const int64_t chunks = std::max<int64_t>(1, ceil_div(R, rpc));
    float* part = static_cast<float*>(ws);
    const int tmb = Mp <= 32 ? 1 : (Mp <= 64 ? 2 : 4), tnb = N <= 32 ? 1 : (N <= 64 ? 2 : 4);
    char label[64];
    snprintf(label, sizeof label, "bwd_dense<bf16>[R%lld,M%lld,N%lld]%s%s", (long long)R, (long long)Mp, (long long)N,
             !Zm ? "nomask" : (mask_bits ? "bits" : ""), dOut ? "" : "dWonly");
    plx_status st;
    {
        KernelTimer kt(ctx, label);
#define PLX_BD(TM, TN)                                                                                                  \
    st = !Zm ? run_bwd<TM, TN, 0>(ctx, R, (int)Mp, (int)N, (const bf16_t*)P, ldp, (const bf16_t*)Q, ldq, nullptr, 0,        \
                                  W, ldw, (bf16_t*)dOut, ldo, part, rpc, chunks)                                        \
         : mask_bits ? run_bwd<TM, TN, 2>(ctx, R, (int)Mp, (int)N, (const bf16_t*)P, ldp, (const bf16_t*)Q, ldq,          \
                                          (const bf16_t*)Zm, ldz, W, ldw, (bf16_t*)dOut, ldo, part, rpc, chunks)        \
                     : run_bwd<TM, TN, 1>(ctx, R, (int)Mp, (int)N, (const bf16_t*)P, ldp, (const bf16_t*)Q, ldq,          \
                                          (const bf16_t*)Zm, ldz, W, ldw, (bf16_t*)dOut, ldo, part, rpc, chunks)
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
