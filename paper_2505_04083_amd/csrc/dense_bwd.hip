// Fused dense part of a GCN layer's backward pass (paper Eq. 2.4, 2.5, 2.6) on the matrix cores.
//
// With Q' = Q * [Zm > 0] (Eq. 2.4; no mask when Zm is NULL) one pass over the rows computes
//     dOut[R x Mp] = Q' W^T          (Eq. 2.6)
//     dW  [Mp x N] = P^T Q'          (Eq. 2.5, reduction over the R rows)
// so the gradient tile Q' is read from HBM once (from its two sources), never written, and
// serves both products from LDS.  P is the aggregated input (aggregate-first order) or the layer
// input (combine-first order); Q is the incoming gradient (or A^T dZ).  All three tall operands
// are streamed exactly once: the kernel is bound by that stream.
//
// Work split: a workgroup (4 wavefronts) owns a chunk of rows and walks it in tiles of 32 rows.
//   dOut tile (32 x Mp): v_mfma_f32_16x16x4_f32; a wavefront owns a few 16-column blocks of dOut and
//       keeps the matching rows of W in registers for the whole kernel (LDS holds only the two
//       row tiles, so several workgroups fit on a CU); lane l supplies a = Q'[row l%16][k + l/16],
//       b = W[16c + l%16][k + l/16] and receives acc[r] = dOut[4*(l/16) + r][16c + l%16].
//   dW (Mp x N): v_mfma_f32_32x32x2_f32 over the 32 rows of the tile, accumulated in registers for
//       the whole chunk; block q of the (Mp/32) x (N/32) grid belongs to wavefront q % 4.
// Chunk partials of dW are summed afterwards in a fixed order (bit-reproducible).
//
// Where both widths exceed 32 the fp32 products are formed from six bf16 matrix products each
// (k_bwd_dense_x3); that kernel can also take the gradient in factored form, Q = G Wn^T with G
// the narrow A^T dZ of a following combine-first layer, and form the tile itself (Eq. 2.6 of
// that layer fused into this pass), so that the R x N gradient never exists in memory.
#include "plx_internal.h"
#include "buffer_addr.h"
#include "bf16_frag.h"

#include <algorithm>

namespace plx {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));


// A kTR x COLS tile held in registers between its global load and its LDS store, so that the
// loads of the next tile are in flight while the matrix cores work on the current one.
template <int TR, int COLS> struct TileRegs { float4 v[TR * COLS / 1024]; };   // TR * COLS / 4 float4 over 256 threads

// Byte offsets of a thread's 16-byte pieces inside a tile, computed once per kernel (VEC path: rows are
// 16-byte aligned, so a piece is one 128-bit buffer load; pieces wholly past the last column get an
// offset no descriptor reaches and read as 0).
template <int TR, int COLS> struct TileOffs { uint32_t v[TR * COLS / 1024]; };

template <int TR, int COLS>
__device__ __forceinline__ void tile_offsets(TileOffs<TR, COLS>& o, int64_t ld, int ncols, int tid) {
    constexpr int Q4 = COLS / 4;
#pragma unroll
    for (int i = 0; i < TR * COLS / 1024; ++i) {
        const int f = tid + 256 * i, r = f / Q4, q = f % Q4;
        o.v[i] = (COLS == ncols || 4 * q < ncols) ? (uint32_t)(((uint32_t)r * (uint32_t)ld + 4u * q) * 4u) : kOutOfRange;
    }
}

// VEC: the tile's descriptor ends with the last column of the last valid row (of the chunk), so rows
// past the end and the bytes behind the matrix read as 0 without any per-lane test.  When ncols is
// not a multiple of 4 the piece that straddles ncols holds padding elements, which are zeroed.
template <int TR, int COLS, bool VEC>
__device__ __forceinline__ void fetch_tile(TileRegs<TR, COLS>& t, const float* __restrict__ src, int64_t ld, int64_t r0,
                                           int64_t r_end, int64_t r_total, int ncols, int tid, const TileOffs<TR, COLS>& o) {
    constexpr int Q4 = COLS / 4;
    if constexpr (VEC) {
        const int64_t left = r_end - r0;
        const int64_t rows = left < TR ? left : TR;
        const __amdgpu_buffer_rsrc_t rs = buffer_of(src + r0 * ld, rows > 0 ? (uint32_t)(((rows - 1) * ld + ncols) * 4) : 0u);
#pragma unroll
        for (int i = 0; i < TR * COLS / 1024; ++i) t.v[i] = buffer_load4(rs, o.v[i]);
        if (ncols & 3) {                               // uniform
#pragma unroll
            for (int i = 0; i < TR * COLS / 1024; ++i) {
                const int gc = 4 * ((tid + 256 * i) % Q4);
                if (gc + 1 >= ncols) t.v[i].y = 0.f;
                if (gc + 2 >= ncols) t.v[i].z = 0.f;
                if (gc + 3 >= ncols) t.v[i].w = 0.f;
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < TR * COLS / 1024; ++i) {
        const int f = tid + 256 * i, r = f / Q4, q = f % Q4;
        const int64_t gr = r0 + r;
        const int gc = 4 * q;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (gr < r_end && gc < ncols) {
            const float* p = src + gr * ld + gc;
            v.x = p[0];
            if (gc + 1 < ncols) v.y = p[1];
            if (gc + 2 < ncols) v.z = p[2];
            if (gc + 3 < ncols) v.w = p[3];
        }
        t.v[i] = v;
    }
}

// How Eq. 2.4 reaches the kernel: no mask, the matrix whose sign decides, or that sign packed one bit per element
enum { kMaskNone = 0, kMaskValues = 1, kMaskBits = 2 };

// Sign bits of a 32-row tile (bit j % 32 of word j / 32 of a row belongs to column j): COLS / 32 words
// per row, 32 * (COLS / 32) words per tile.  Chunk i of thread tid (4 columns) lies in word
// tid / 8 + 32 i of the tile, so a wavefront needs only 8 words per i: lane l < 8 * (COLS / 32) loads
// word 8 * wavefront + l % 8 + 32 * (l / 8), and at commit time chunk i takes its word from lane
// l / 8 + 8 i with a cross-lane read and its nibble at bit 4 * (tid % 8).
template <int TR, int COLS> struct TileBits { uint32_t w; };

template <int TR, int COLS>
__device__ __forceinline__ uint32_t bits_offset(int64_t ldbits, int ncols, int tid) {      // byte offset of a lane's word in a tile
    static_assert(TR == 32, "word numbering assumes 32-row tiles");
    constexpr int WPR = COLS / 32;
    const int lane = tid & 63, wv = tid >> 6;
    const int wi = 8 * wv + (lane & 7) + 32 * (lane >> 3);
    const int cw = wi % WPR;
    return (lane < 8 * WPR && 32 * cw < ncols) ? (uint32_t)(((uint32_t)(wi / WPR) * (uint32_t)ldbits + cw) * 4u) : kOutOfRange;
}

template <int TR, int COLS>
__device__ __forceinline__ void fetch_bits(TileBits<TR, COLS>& t, const uint32_t* __restrict__ bits, int64_t ldbits,
                                           int64_t r0, int64_t r_end, int ncols, uint32_t off) {
    const int64_t left = r_end - r0;
    const int64_t rows = left < TR ? left : TR;
    const __amdgpu_buffer_rsrc_t rs = buffer_of(bits + r0 * ldbits, rows > 0 ? (uint32_t)(((rows - 1) * ldbits + (ncols + 31) / 32) * 4) : 0u);
    t.w = buffer_load1(rs, off);
}

// registers -> LDS tile [TR][COLS + 4]; with a mask, elements whose mask is <= 0 (whose bit is clear) become 0 (Eq. 2.4)
template <int TR, int COLS, int MASK>
__device__ __forceinline__ void commit_tile(float (*dst)[COLS + 4], const TileRegs<TR, COLS>& t,
                                            const TileRegs<TR, COLS>& m, const TileBits<TR, COLS>& mb, int tid) {
    constexpr int Q4 = COLS / 4;
#pragma unroll
    for (int i = 0; i < TR * COLS / 1024; ++i) {
        const int f = tid + 256 * i, r = f / Q4, q = f % Q4;
        float4 v = t.v[i];
        if (MASK == kMaskValues) {
            const float4 z = m.v[i];
            v.x = z.x > 0.f ? v.x : 0.f; v.y = z.y > 0.f ? v.y : 0.f;
            v.z = z.z > 0.f ? v.z : 0.f; v.w = z.w > 0.f ? v.w : 0.f;
        } else if (MASK == kMaskBits) {
            // bit e of the nibble, sign-extended to a word mask: two vector instructions per element
            const int b = (int)__shfl(mb.w, ((tid & 63) >> 3) + 8 * i);
            const unsigned s0 = 4 * (tid & 7);
            v.x = __uint_as_float(__float_as_uint(v.x) & (unsigned)__builtin_amdgcn_sbfe(b, s0, 1));
            v.y = __uint_as_float(__float_as_uint(v.y) & (unsigned)__builtin_amdgcn_sbfe(b, s0 + 1, 1));
            v.z = __uint_as_float(__float_as_uint(v.z) & (unsigned)__builtin_amdgcn_sbfe(b, s0 + 2, 1));
            v.w = __uint_as_float(__float_as_uint(v.w) & (unsigned)__builtin_amdgcn_sbfe(b, s0 + 3, 1));
        }
        *reinterpret_cast<float4*>(&dst[r][4 * q]) = v;
    }
}

constexpr int kTR = 32;      // rows per tile

template <int TMB, int TNB, int MASK, bool VEC>   // Mp <= 32*TMB, N <= 32*TNB; with kMaskBits Zm points at words
__global__ __launch_bounds__(256) void k_bwd_dense_f32(int64_t R, int Mp, int N, const float* __restrict__ P, int64_t ldp,
                                                       const float* __restrict__ Q, int64_t ldq,
                                                       const float* __restrict__ Zm, int64_t ldz,
                                                       const float* __restrict__ W, int64_t ldw,
                                                       float* __restrict__ dOut, int64_t ldo, float* __restrict__ part,
                                                       int64_t rows_per_chunk) {
    constexpr int MP = 32 * TMB, NP = 32 * TNB;
    // dW blocks over 4 wavefronts: NB >= 4 gives NB/4 blocks each; with NB < 4 the 4/NB wavefronts
    // sharing a block take interleaved row pairs of every tile and write separate partial tiles.
    constexpr int NB = TMB * TNB, KS = NB >= 4 ? 1 : 4 / NB, NBLK = NB >= 4 ? NB / 4 : 1;
    // dOut tile = 2 x NCB blocks of 16x16.  A wavefront owns NCW column blocks (and with them NCW
    // slices of W, kept in registers as ready-made B operands for the whole kernel) of NRW row blocks:
    // Mp >= 64: column blocks w*NCW.., both row blocks; Mp <= 32: column block w/2 of row block w%2.
    constexpr int NCB = MP / 16, NCW = NCB >= 4 ? NCB / 4 : 1, NRW = NCB >= 4 ? 2 : 1;
    constexpr int NKS = NP / 4, CHUNK = 8;
    extern __shared__ __align__(16) float smem[];
    float (*Qs)[NP + 4] = reinterpret_cast<float (*)[NP + 4]>(smem);
    float (*Ps)[MP + 4] = reinterpret_cast<float (*)[MP + 4]>(smem + kTR * (NP + 4));

    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5, l16 = lane & 15, lq = lane >> 4;
    const int wq = NB >= 4 ? w : w % NB, ks = NB >= 4 ? 0 : w / NB;
    const int cb0 = NCB >= 4 ? w * NCW : (w >> 1), rb0 = NCB >= 4 ? 0 : (w & 1);
    const int n_end = (N + 3) & ~3;
    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_chunk;
    const int64_t r_end = (r_begin + rows_per_chunk < R) ? r_begin + rows_per_chunk : R;

    float wreg[NCW][NKS];                  // wreg[c][s] = W[16*(cb0+c) + l%16][4s + l/16]
#pragma unroll
    for (int c = 0; c < NCW; ++c) {
        const int i = 16 * (cb0 + c) + l16;
#pragma unroll
        for (int s2 = 0; s2 < NKS; ++s2) {
            const int n = 4 * s2 + lq;
            wreg[c][s2] = (dOut && i < Mp && n < N) ? W[(int64_t)i * ldw + n] : 0.f;
        }
    }
    // the weights must have landed before the row loop: otherwise their first use inside the loop
    // would wait for all outstanding loads, the prefetch of the next tile included
    __builtin_amdgcn_s_waitcnt(0x0F70);    // vmcnt(0), other counters untouched

    floatx16 acc_w[NBLK];
#pragma unroll
    for (int t = 0; t < NBLK; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_w[t][r] = 0.f;

    // Order inside an iteration: issue the next tile's global loads, run both products from LDS,
    // barrier, write the prefetched tile to LDS, and only then issue this tile's dOut stores.
    TileRegs<kTR, NP> rq, rz;
    TileRegs<kTR, MP> rp;
    TileBits<kTR, NP> zb;
    TileBits<kTR, MP> nb;                  // never read
    TileOffs<kTR, NP> oq, oz;
    TileOffs<kTR, MP> op;
    tile_offsets<kTR, NP>(oq, ldq, N, tid);
    if (MASK == kMaskValues) tile_offsets<kTR, NP>(oz, ldz, N, tid);
    tile_offsets<kTR, MP>(op, ldp, Mp, tid);
    const uint32_t* Zbits = reinterpret_cast<const uint32_t*>(Zm);
    const uint32_t ob = MASK == kMaskBits ? bits_offset<kTR, NP>(ldz, N, tid) : 0u;
    fetch_tile<kTR, NP, VEC>(rq, Q, ldq, r_begin, r_end, R, N, tid, oq);
    if (MASK == kMaskValues) fetch_tile<kTR, NP, VEC>(rz, Zm, ldz, r_begin, r_end, R, N, tid, oz);
    if (MASK == kMaskBits) fetch_bits<kTR, NP>(zb, Zbits, ldz, r_begin, r_end, N, ob);
    fetch_tile<kTR, MP, VEC>(rp, P, ldp, r_begin, r_end, R, Mp, tid, op);
    commit_tile<kTR, NP, MASK>(Qs, rq, rz, zb, tid);
    commit_tile<kTR, MP, kMaskNone>(Ps, rp, rp, nb, tid);
    __syncthreads();

    for (int64_t r0 = r_begin; r0 < r_end; r0 += kTR) {
        // No condition around the prefetch and its LDS write (the last pass re-reads its own tile):
        // with straight-line code the only wait for loads sits right before the LDS write and
        // nothing waits for the previous tile's stores to be acknowledged.
        const int64_t rn = r0 + kTR < r_end ? r0 + kTR : r0;
        fetch_tile<kTR, NP, VEC>(rq, Q, ldq, rn, r_end, R, N, tid, oq);
        if (MASK == kMaskValues) fetch_tile<kTR, NP, VEC>(rz, Zm, ldz, rn, r_end, R, N, tid, oz);
        if (MASK == kMaskBits) fetch_bits<kTR, NP>(zb, Zbits, ldz, rn, r_end, N, ob);
        fetch_tile<kTR, MP, VEC>(rp, P, ldp, rn, r_end, R, Mp, tid, op);

        floatx4 acc_o[NRW][NCW];
        if (dOut) {                                                    // Eq. 2.6 on this tile
#pragma unroll
            for (int rr = 0; rr < NRW; ++rr)
#pragma unroll
                for (int c = 0; c < NCW; ++c) acc_o[rr][c] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s0 = 0; s0 < NKS; s0 += CHUNK) {
                if (4 * s0 >= n_end) break;                            // uniform: no matrix work on padding beyond a chunk
#pragma unroll
                for (int s2 = s0; s2 < s0 + CHUNK; ++s2) {
                    float a[NRW];
#pragma unroll
                    for (int rr = 0; rr < NRW; ++rr) a[rr] = Qs[16 * (rb0 + rr) + l16][4 * s2 + lq];
#pragma unroll
                    for (int rr = 0; rr < NRW; ++rr)
#pragma unroll
                        for (int c = 0; c < NCW; ++c)
                            acc_o[rr][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[rr], wreg[c][s2], acc_o[rr][c], 0, 0, 0);
                }
            }
        }
#pragma unroll 4
        for (int kk = 2 * ks; kk < kTR; kk += 2 * KS) {                // Eq. 2.5, partial over this tile
#pragma unroll
            for (int t = 0; t < NBLK; ++t) {
                const int q = wq + 4 * t, bi = q / TNB, bj = q % TNB;
                acc_w[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(Ps[kk + lh][32 * bi + l32], Qs[kk + lh][32 * bj + l32],
                                                                acc_w[t], 0, 0, 0);
            }
        }
        __syncthreads();                                               // every wavefront is done reading the tile
        commit_tile<kTR, NP, MASK>(Qs, rq, rz, zb, tid);
        commit_tile<kTR, MP, kMaskNone>(Ps, rp, rp, nb, tid);
        if (dOut) {
            const bool full = r0 + kTR <= r_end;                       // uniform: only the last tile is partial
            const __amdgpu_buffer_rsrc_t ro = buffer_of(dOut + r0 * ldo, (uint32_t)(((kTR - 1) * ldo + Mp) * 4));
#pragma unroll
            for (int rr = 0; rr < NRW; ++rr) {
                const int row0 = 16 * (rb0 + rr);                      // uniform; the lane's rows are row0 + 4*lq + r
                uint32_t orow = opaque_zero() + (uint32_t)row0 * (uint32_t)ldo * 4u;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
#pragma unroll
                    for (int c = 0; c < NCW; ++c) {
                        const int gc = 16 * (cb0 + c) + l16;
                        const uint32_t ooff = gc < Mp ? (uint32_t)((4u * lq * (uint32_t)ldo + gc) * 4u) : kOutOfRange;
                        if (full || r0 + row0 + 4 * lq + r < r_end) buffer_store(ro, ooff, orow, acc_o[rr][c][r]);
                    }
                    orow += (uint32_t)ldo * 4u;
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

// ---- the same pass with the fp32 products taken through the bf16 matrix instructions ----------------
// An fp32 value is the exact sum of three bf16 numbers (each rounded to nearest even from what the
// others leave: 8 + 8 + 8 significand bits), and a product of two bf16 numbers is exact in fp32.
// With a = a1 + a2 + a3 and b = b1 + b2 + b3, the six products a1 b1, a1 b2, a2 b1, a2 b2, a1 b3,
// a3 b1 carry a b up to terms below 2^-23 |a b|, i.e. to fp32 rounding; accumulation is fp32 inside
// the matrix instruction as before.  Six bf16 instructions cover 16 (32) values of k in the time the
// fp32 instruction needs for 3 (6): where the fp32 matrix pipe binds (both widths 64 or more) this
// path is taken instead (an infinite input gives NaN here, inf - inf, where the plain product gives inf).
// The tiles are split once, when they are written to LDS as three bf16 planes.
#ifndef PLX_X3_PAD
#define PLX_X3_PAD 16         // padding of an LDS row of a bf16 plane, in elements (a multiple of 8 keeps rows 16-byte aligned; 16 measured 1-4 % faster than 8: fewer bank conflicts of the transpose reads)
#endif
// registers -> three bf16 planes of an LDS tile [3][TR][COLS + 8], masked like commit_tile
template <int TR, int COLS, int MASK>
__device__ __forceinline__ void commit_split(bf16_t* dst, const TileRegs<TR, COLS>& t, const TileRegs<TR, COLS>& m,
                                             const TileBits<TR, COLS>& mb, int tid) {
    constexpr int Q4 = COLS / 4, PITCH = COLS + PLX_X3_PAD, PLANE = TR * PITCH;
#pragma unroll
    for (int i = 0; i < TR * COLS / 1024; ++i) {
        const int f = tid + 256 * i, r = f / Q4, q = f % Q4;
        float4 v = t.v[i];
        if (MASK == kMaskValues) {
            const float4 z = m.v[i];
            v.x = z.x > 0.f ? v.x : 0.f; v.y = z.y > 0.f ? v.y : 0.f;
            v.z = z.z > 0.f ? v.z : 0.f; v.w = z.w > 0.f ? v.w : 0.f;
        } else if (MASK == kMaskBits) {
            const int b = (int)__shfl(mb.w, ((tid & 63) >> 3) + 8 * i);
            const unsigned s0 = 4 * (tid & 7);
            v.x = __uint_as_float(__float_as_uint(v.x) & (unsigned)__builtin_amdgcn_sbfe(b, s0, 1));
            v.y = __uint_as_float(__float_as_uint(v.y) & (unsigned)__builtin_amdgcn_sbfe(b, s0 + 1, 1));
            v.z = __uint_as_float(__float_as_uint(v.z) & (unsigned)__builtin_amdgcn_sbfe(b, s0 + 2, 1));
            v.w = __uint_as_float(__float_as_uint(v.w) & (unsigned)__builtin_amdgcn_sbfe(b, s0 + 3, 1));
        }
        uint2 pl[3];
        split3(v, pl);
#pragma unroll
        for (int p = 0; p < 3; ++p) *reinterpret_cast<uint2*>(dst + p * PLANE + r * PITCH + 4 * q) = pl[p];
    }
}

#ifndef PLX_X3_BWD_WAVES
#define PLX_X3_BWD_WAVES 2
#endif
// Wavefronts per SIMD the register allocation aims at.  The 64 x 128 kernel with a factored gradient fits three with
// five spilled registers and gains 3.5 % from the third wavefront (road network, 50 M rows); the 128-wide kernels would
// spill over a hundred registers at three (measured 2.2 times slower) and stay at two.
constexpr int x3_bwd_waves(int tmb, int tnb, int dns) { return (tmb == 2 && tnb == 4 && dns == 1) ? 3 : PLX_X3_BWD_WAVES; }

// DNS > 0: the gradient arrives in factored form, Q = Gf Wn^T with Gf[R x dn] and Wn[N x dn], dn <= 16*DNS (the
// following combine-first layer's A^T dZ and its weights, Eq. 2.6 of that layer; DNS <= 2): the 32 x N tile of Q is formed
// here, by the same split products, and goes straight to LDS, so the R x N gradient is neither written by
// that layer nor read by this one.  Wavefront w forms columns 32w .. 32w+31 (TNB == 4) as Q^T = Wn Gf^T, which
// leaves a lane with four consecutive columns of one row per group of accumulator registers: the layout
// the masking and the split already work on.  Mask: none or sign bits.
template <int TMB, int TNB, int MASK, int DNS>   // 64 <= Mp <= 32*TMB, 64 <= N <= 32*TNB (TMB, TNB in {2, 4}); 16-byte aligned rows
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(x3_bwd_waves(TMB, TNB, DNS)))) void k_bwd_dense_x3(int64_t R, int Mp, int N, const float* __restrict__ P, int64_t ldp,
                                                      const float* __restrict__ Q, int64_t ldq,
                                                      const float* __restrict__ Zm, int64_t ldz,
                                                      const float* __restrict__ W, int64_t ldw,
                                                      float* __restrict__ dOut, int64_t ldo, float* __restrict__ part,
                                                      int64_t rows_per_chunk, const float* __restrict__ Gf, int64_t ldg,
                                                      const float* __restrict__ Wn, int64_t ldwn, int dn) {
    constexpr bool FACT = DNS > 0;
    static_assert(!FACT || (TNB == 4 && MASK != kMaskValues), "shapes of the factored gradient");
    constexpr int MP = 32 * TMB, NP = 32 * TNB, SQ = NP + PLX_X3_PAD, SP = MP + PLX_X3_PAD;
    constexpr int NBLK = TMB * TNB / 4;                       // 32x32 blocks of dW per wavefront (block q belongs to wavefront q % 4)
    constexpr int NCW = MP / 64, NRW = kTR / 16, NKS = NP / 32;   // dOut: NCW column blocks of 16 per wavefront, both row blocks
    static_assert(TMB >= 2 && TNB >= 2 && kTR == 32, "shapes of the split path");
    extern __shared__ __align__(16) unsigned char smem_raw[];
    bf16_t* Qs = reinterpret_cast<bf16_t*>(smem_raw);         // [3][kTR][SQ]
    bf16_t* Ps = Qs + 3 * kTR * SQ;                           // [3][kTR][SP]
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5, l16 = lane & 15, lq = lane >> 4;
    const int cb0 = w * NCW;
    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_chunk;
    const int64_t r_end = (r_begin + rows_per_chunk < R) ? r_begin + rows_per_chunk : R;

    bf16x8 wreg[NCW][NKS][3];              // planes of W[16*(cb0+c) + l16][32s + 8*lq .. +7]
#pragma unroll
    for (int c = 0; c < NCW; ++c) {
        const int i = 16 * (cb0 + c) + l16;
#pragma unroll
        for (int s2 = 0; s2 < NKS; ++s2) {
            Frag f[3];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int n = 32 * s2 + 8 * lq + 4 * h;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (dOut && i < Mp) {
                    const float* wp = W + (int64_t)i * ldw + n;
                    if (n < N) v.x = wp[0];
                    if (n + 1 < N) v.y = wp[1];
                    if (n + 2 < N) v.z = wp[2];
                    if (n + 3 < N) v.w = wp[3];
                }
                uint2 pl[3];
                split3<true>(v, pl);
#pragma unroll
                for (int p = 0; p < 3; ++p) { f[p].x[2 * h] = pl[p].x; f[p].x[2 * h + 1] = pl[p].y; }
            }
#pragma unroll
            for (int p = 0; p < 3; ++p) wreg[c][s2][p] = f[p].v;
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);    // weights landed before the row loop (vmcnt(0))

    floatx16 acc_w[NBLK];
#pragma unroll
    for (int t = 0; t < NBLK; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_w[t][r] = 0.f;

    TileRegs<kTR, NP> rq, rz;
    TileRegs<kTR, MP> rp;
    TileBits<kTR, NP> zb;
    TileBits<kTR, MP> nb;                  // never read
    TileOffs<kTR, NP> oq, oz;
    TileOffs<kTR, MP> op;
    if (!FACT) tile_offsets<kTR, NP>(oq, ldq, N, tid);
    if (MASK == kMaskValues) tile_offsets<kTR, NP>(oz, ldz, N, tid);
    tile_offsets<kTR, MP>(op, ldp, Mp, tid);
    const uint32_t* Zbits = reinterpret_cast<const uint32_t*>(Zm);
    const uint32_t ob = (MASK == kMaskBits && !FACT) ? bits_offset<kTR, NP>(ldz, N, tid) : 0u;

    // factored gradient: planes of Wn[32w + l32][16s + 8*lh .. +7] for the whole kernel; per tile a lane fetches
    // Gf[row l32][16s + 8*lh .. +7] (two 16-byte pieces per s) and the sign word of (row l32, columns 32w ..)
    constexpr int NS = FACT ? DNS : 1;
    bf16x8 wnreg[NS][3];
    uint32_t goff[NS][2];
    float4 gq[NS][2];
    uint32_t zw = 0;
    const uint32_t zoff = (FACT && MASK == kMaskBits && 32 * w < N) ? (uint32_t)(((uint32_t)l32 * (uint32_t)ldz + w) * 4u) : kOutOfRange;
    if constexpr (FACT) {
        const int n = 32 * w + l32;
#pragma unroll
        for (int s2 = 0; s2 < NS; ++s2) {
            Frag f[3];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int k = 16 * s2 + 8 * lh + 4 * h;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (n < N) {
                    const float* wp = Wn + (int64_t)n * ldwn + k;
                    if (k < dn) v.x = wp[0];
                    if (k + 1 < dn) v.y = wp[1];
                    if (k + 2 < dn) v.z = wp[2];
                    if (k + 3 < dn) v.w = wp[3];
                }
                uint2 pl[3];
                split3<true>(v, pl);
#pragma unroll
                for (int p = 0; p < 3; ++p) { f[p].x[2 * h] = pl[p].x; f[p].x[2 * h + 1] = pl[p].y; }
                goff[s2][h] = k < dn ? (uint32_t)(((uint32_t)l32 * (uint32_t)ldg + k) * 4u) : kOutOfRange;
            }
#pragma unroll
            for (int p = 0; p < 3; ++p) wnreg[s2][p] = f[p].v;
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);
    }
    auto fetch = [&](int64_t r0) {
        if constexpr (FACT) {
            const int64_t left = r_end - r0;
            const int64_t rows = left < kTR ? left : kTR;
            const __amdgpu_buffer_rsrc_t rg = buffer_of(Gf + r0 * ldg, rows > 0 ? (uint32_t)(((rows - 1) * ldg + dn) * 4) : 0u);
#pragma unroll
            for (int s2 = 0; s2 < NS; ++s2)
#pragma unroll
                for (int h = 0; h < 2; ++h) gq[s2][h] = buffer_load4(rg, goff[s2][h]);
            if (MASK == kMaskBits) {
                const __amdgpu_buffer_rsrc_t rb = buffer_of(Zbits + r0 * ldz, rows > 0 ? (uint32_t)(((rows - 1) * ldz + (N + 31) / 32) * 4) : 0u);
                zw = buffer_load1(rb, zoff);
            }
        } else {
            fetch_tile<kTR, NP, true>(rq, Q, ldq, r0, r_end, R, N, tid, oq);
            if (MASK == kMaskValues) fetch_tile<kTR, NP, true>(rz, Zm, ldz, r0, r_end, R, N, tid, oz);
            if (MASK == kMaskBits) fetch_bits<kTR, NP>(zb, Zbits, ldz, r0, r_end, N, ob);
        }
        fetch_tile<kTR, MP, true>(rp, P, ldp, r0, r_end, R, Mp, tid, op);
    };
    // registers -> the three planes of the (masked) gradient tile in LDS
    auto commit_q = [&]() {
        if constexpr (FACT) {
            floatx16 qt;
#pragma unroll
            for (int r = 0; r < 16; ++r) qt[r] = 0.f;
#pragma unroll
            for (int s2 = 0; s2 < NS; ++s2) {
                if (s2 > 0 && 16 * s2 >= dn) break;                          // uniform
                Frag f[3];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    float4 v = gq[s2][h];
                    if (dn & 3) {                                            // uniform: the piece that straddles dn holds padding
                        const int k = 16 * s2 + 8 * lh + 4 * h;
                        if (k + 1 >= dn) v.y = 0.f;
                        if (k + 2 >= dn) v.z = 0.f;
                        if (k + 3 >= dn) v.w = 0.f;
                    }
                    uint2 pl[3];
                    split3(v, pl);
#pragma unroll
                    for (int p = 0; p < 3; ++p) { f[p].x[2 * h] = pl[p].x; f[p].x[2 * h + 1] = pl[p].y; }
                }
                bf16x8 b[3] = {f[0].v, f[1].v, f[2].v};
                PLX_X3_32(qt, wnreg[s2], b);                                 // qt[r] = Q[row l32][32w + 8*(r/4) + 4*lh + r%4]
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float4 v = make_float4(qt[4 * g], qt[4 * g + 1], qt[4 * g + 2], qt[4 * g + 3]);
                if (MASK == kMaskBits) {
                    const unsigned s0 = 8 * g + 4 * lh;
                    v.x = __uint_as_float(__float_as_uint(v.x) & (unsigned)__builtin_amdgcn_sbfe((int)zw, s0, 1));
                    v.y = __uint_as_float(__float_as_uint(v.y) & (unsigned)__builtin_amdgcn_sbfe((int)zw, s0 + 1, 1));
                    v.z = __uint_as_float(__float_as_uint(v.z) & (unsigned)__builtin_amdgcn_sbfe((int)zw, s0 + 2, 1));
                    v.w = __uint_as_float(__float_as_uint(v.w) & (unsigned)__builtin_amdgcn_sbfe((int)zw, s0 + 3, 1));
                }
                uint2 pl[3];
                split3(v, pl);
#pragma unroll
                for (int p = 0; p < 3; ++p) *reinterpret_cast<uint2*>(Qs + p * kTR * SQ + l32 * SQ + 32 * w + 8 * g + 4 * lh) = pl[p];
            }
        } else {
            commit_split<kTR, NP, MASK>(Qs, rq, rz, zb, tid);
        }
    };
    fetch(r_begin);
    commit_q();
    commit_split<kTR, MP, kMaskNone>(Ps, rp, rp, nb, tid);
    __syncthreads();

    const int n_end = (N + 31) & ~31;
    for (int64_t r0 = r_begin; r0 < r_end; r0 += kTR) {
        fetch(r0 + kTR < r_end ? r0 + kTR : r0);                       // unconditional: the last pass re-reads its own tile

        floatx4 acc_o[NRW][NCW];
        if (dOut) {                                                    // Eq. 2.6 on this tile
#pragma unroll
            for (int rr = 0; rr < NRW; ++rr)
#pragma unroll
                for (int c = 0; c < NCW; ++c) acc_o[rr][c] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s2 = 0; s2 < NKS; ++s2) {
                if (32 * s2 >= n_end) break;                           // uniform
#pragma unroll
                for (int rr = 0; rr < NRW; ++rr) {
                    bf16x8 a[3];
#pragma unroll
                    for (int p = 0; p < 3; ++p) a[p] = frag_contig(Qs + p * kTR * SQ + (16 * rr + l16) * SQ + 32 * s2 + 8 * lq);
#pragma unroll
                    for (int c = 0; c < NCW; ++c) PLX_X3_16(acc_o[rr][c], a, wreg[c][s2]);
                }
            }
        }
#pragma unroll
        for (int kk = 0; kk < kTR; kk += 16) {                         // Eq. 2.5: 16 rows of the tile per instruction
            bf16x8 b[3];                                               // 4 % TNB == 0: all blocks of a wavefront share the column block w % TNB
#pragma unroll
            for (int p = 0; p < 3; ++p) b[p] = frag_column(Qs + p * kTR * SQ, SQ, kk, 32 * (w % TNB), lane);
#pragma unroll
            for (int t = 0; t < NBLK; ++t) {
                const int bi = (w + 4 * t) / TNB;
                bf16x8 a[3];
#pragma unroll
                for (int p = 0; p < 3; ++p) a[p] = frag_column(Ps + p * kTR * SP, SP, kk, 32 * bi, lane);
                PLX_X3_32(acc_w[t], a, b);
            }
        }
        __syncthreads();                                               // every wavefront is done reading the tile
        commit_q();
        commit_split<kTR, MP, kMaskNone>(Ps, rp, rp, nb, tid);
        if (dOut) {
            const bool full = r0 + kTR <= r_end;                       // uniform: only the last tile is partial
            const __amdgpu_buffer_rsrc_t ro = buffer_of(dOut + r0 * ldo, (uint32_t)(((kTR - 1) * ldo + Mp) * 4));
#pragma unroll
            for (int rr = 0; rr < NRW; ++rr) {
                const int row0 = 16 * rr;                              // uniform; the lane's rows are row0 + 4*lq + r
                uint32_t orow = opaque_zero() + (uint32_t)row0 * (uint32_t)ldo * 4u;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
#pragma unroll
                    for (int c = 0; c < NCW; ++c) {
                        const int gc = 16 * (cb0 + c) + l16;
                        const uint32_t ooff = gc < Mp ? (uint32_t)((4u * lq * (uint32_t)ldo + gc) * 4u) : kOutOfRange;
                        if (full || r0 + row0 + 4 * lq + r < r_end) buffer_store(ro, ooff, orow, acc_o[rr][c][r]);
                    }
                    orow += (uint32_t)ldo * 4u;
                }
            }
        }
        __syncthreads();
    }

    float* out = part + (int64_t)blockIdx.x * Mp * N;
#pragma unroll
    for (int t = 0; t < NBLK; ++t) {
        const int q = w + 4 * t, bi = q / TNB, bj = q % TNB;
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

// the gradient in factored form, Q = G Wn^T (G: R x dn, Wn: N x dn); G == NULL: Q is given
struct Factor {
    const float* G = nullptr;
    int64_t ldg = 0;
    const float* Wn = nullptr;
    int64_t ldwn = 0;
    int dn = 0;
};

template <int TMB, int TNB, int MASK>
plx_status run_masked(plx_ctx* ctx, int64_t R, int Mp, int N, const float* P, int64_t ldp, const float* Q, int64_t ldq,
                      const float* Zm, int64_t ldz, const float* W, int64_t ldw, float* dOut, int64_t ldo, float* part,
                      int64_t rpc, int64_t chunks, bool vec, bool split, const Factor& fac) {
    constexpr int MP = 32 * TMB, NP = 32 * TNB;
    const size_t lds = sizeof(float) * (kTR * (NP + 4) + kTR * (MP + 4));
    if constexpr (TMB >= 2 && TNB >= 2) {
        if (split) {                                                     // both widths above 32: the fp32 matrix pipe binds
            const size_t lds3 = sizeof(bf16_t) * 3 * kTR * ((NP + PLX_X3_PAD) + (MP + PLX_X3_PAD));
            auto launch3 = [&](auto kern) -> plx_status {
                if (lds3 > 48 * 1024)
                    PLX_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds3));
                kern<<<dim3((unsigned)chunks), 256, lds3, ctx->stream>>>(R, Mp, N, P, ldp, Q, ldq, Zm, ldz, W, ldw, dOut, ldo, part, rpc,
                                                                        fac.G, fac.ldg, fac.Wn, fac.ldwn, fac.dn);
                PLX_HIP(ctx, hipGetLastError());
                return PLX_OK;
            };
            if (fac.G) {
                if constexpr (TNB == 4 && MASK != kMaskValues) {
                    if (fac.dn <= 16) return launch3(k_bwd_dense_x3<TMB, TNB, MASK, 1>);
                    return launch3(k_bwd_dense_x3<TMB, TNB, MASK, 2>);
                }
                return fail(ctx, PLX_ERR_INTERNAL, "factored gradient outside the fused kernel's range");
            }
            return launch3(k_bwd_dense_x3<TMB, TNB, MASK, 0>);
        }
    }
    if (fac.G) return fail(ctx, PLX_ERR_INTERNAL, "factored gradient outside the fused kernel's range");
    auto launch = [&](auto kern) -> plx_status {
        kern<<<dim3((unsigned)chunks), 256, lds, ctx->stream>>>(R, Mp, N, P, ldp, Q, ldq, Zm, ldz, W, ldw, dOut, ldo, part, rpc);
        PLX_HIP(ctx, hipGetLastError());
        return PLX_OK;
    };
    return vec ? launch(k_bwd_dense_f32<TMB, TNB, MASK, true>) : launch(k_bwd_dense_f32<TMB, TNB, MASK, false>);
}

template <int TMB, int TNB>
plx_status run(plx_ctx* ctx, int64_t R, int Mp, int N, const float* P, int64_t ldp, const float* Q, int64_t ldq,
               const float* Zm, int64_t ldz, const float* W, int64_t ldw, float* dOut, int64_t ldo, float* part,
               int64_t rpc, int64_t chunks, bool mask_bits, bool vec, bool split, const Factor& fac) {
    if (!Zm) return run_masked<TMB, TNB, kMaskNone>(ctx, R, Mp, N, P, ldp, Q, ldq, Zm, ldz, W, ldw, dOut, ldo, part, rpc, chunks, vec, split, fac);
    return mask_bits ? run_masked<TMB, TNB, kMaskBits>(ctx, R, Mp, N, P, ldp, Q, ldq, Zm, ldz, W, ldw, dOut, ldo, part, rpc, chunks, vec, split, fac)
                     : run_masked<TMB, TNB, kMaskValues>(ctx, R, Mp, N, P, ldp, Q, ldq, Zm, ldz, W, ldw, dOut, ldo, part, rpc, chunks, vec, split, fac);
}

}  // namespace

bool bwd_dense_supported(int64_t Mp, int64_t N, plx_dtype dtype) { return (dtype == PLX_F32 || dtype == PLX_BF16) && Mp <= 128 && N <= 128; }

// Can the fused kernel form its gradient tile from the factors G[R x dn] Wn[N x dn]^T itself?  Only the split fp32
// kernel with four column blocks does (64 < N <= 128, 32 < Mp <= 128, no value mask, 16-byte aligned rows), and
// only for dn <= 32: every 16 values of dn add six matrix instructions and two splits per tile and 12 registers
// to a kernel that is bound by exactly those (measured: dn = 47, four steps, spills and doubles the kernel's time).
bool bwd_dense_factor_supported(const plx_ctx* ctx, int64_t R, int64_t Mp, int64_t N, int64_t dn, plx_dtype dtype, const void* P,
                                int64_t ldp, const void* G, int64_t ldg, int64_t ldz, int64_t ldo, bool value_mask) {
    return dtype == PLX_F32 && ctx->split_products && R > 0 && Mp > 32 && Mp <= 128 && N > 64 && N <= 128 && dn > 0 && dn <= 32 &&
           !value_mask && aligned16(P) && ldp % 4 == 0 && aligned16(G) && ldg % 4 == 0 &&
           std::max(std::max(ldp, ldg), std::max(ldz, ldo)) < (int64_t(1) << 23);
}

plx_status launch_bwd_dense(plx_ctx* ctx, int64_t R, int64_t Mp, int64_t N, const void* P, int64_t ldp, const void* Q,
                            int64_t ldq, const void* Zm, int64_t ldz, const float* W, int64_t ldw, void* dOut, int64_t ldo,
                            float* dW, int64_t lddw, plx_dtype dtype, void* ws, size_t ws_bytes, bool mask_bits,
                            const float* G, int64_t ldg, const float* Wn, int64_t ldwn, int64_t dn) {
    if (!bwd_dense_supported(Mp, N, dtype)) return fail(ctx, PLX_ERR_INTERNAL, "fused backward called outside its range");
    // a tile is addressed with 31-bit byte offsets: 32 rows * ld * 4 bytes must fit
    if (std::max(std::max(ldp, ldq), std::max(ldz, ldo)) >= (int64_t(1) << 23))
        return fail(ctx, PLX_ERR_UNSUPPORTED, "leading dimensions of 2^23 elements or more are not supported by the fused backward kernels");
    if (G && !bwd_dense_factor_supported(ctx, R, Mp, N, dn, dtype, P, ldp, G, ldg, ldz, ldo, Zm && !mask_bits))
        return fail(ctx, PLX_ERR_INTERNAL, "factored gradient outside the fused kernel's range");
    if (dtype == PLX_BF16)
        return launch_bwd_dense_bf16(ctx, R, Mp, N, P, ldp, Q, ldq, Zm, ldz, W, ldw, dOut, ldo, dW, lddw, ws, ws_bytes, mask_bits);
    if (ws_bytes < gemm_tn_workspace(R, Mp, N)) return fail(ctx, PLX_ERR_SHAPE, "workspace too small");
    const int64_t rpc = tn_rows_per_chunk(R, Mp, N);
    const int64_t chunks = std::max<int64_t>(1, ceil_div(R, rpc));
    float* part = static_cast<float*>(ws);
    const int tmb = Mp <= 32 ? 1 : (Mp <= 64 ? 2 : 4), tnb = N <= 32 ? 1 : (N <= 64 ? 2 : 4);
    char label[64];
    // 128-bit tile loads need 16-byte aligned rows; the split path (six bf16 products per fp32 product) serves the
    // shapes whose fp32 matrix work binds, i.e. both widths above 32
    const bool values = Zm && !mask_bits;
    const bool vec = aligned16(P) && ldp % 4 == 0 && (G || (aligned16(Q) && ldq % 4 == 0)) && (!values || (aligned16(Zm) && ldz % 4 == 0)) && R > 0;
    const bool split = vec && ctx->split_products && tmb >= 2 && tnb >= 2;
    Factor fac;
    fac.G = G; fac.ldg = ldg; fac.Wn = Wn; fac.ldwn = ldwn; fac.dn = (int)dn;
    char fact[16] = "";
    if (G) snprintf(fact, sizeof fact, "fact%lld", (long long)dn);
    // suffixes: x3 split products, bits / nomask how Eq. 2.4 arrives (default: a value matrix), fact<dn> factored gradient,
    // dWonly Eq. 2.6 not wanted
    snprintf(label, sizeof label, "bwd_dense<f32>[R%lld,M%lld,N%lld]%s%s%s%s", (long long)R, (long long)Mp, (long long)N,
             split ? "x3" : "", !Zm ? "nomask" : (mask_bits ? "bits" : ""), fact, dOut ? "" : "dWonly");
    plx_status st;
    {
        KernelTimer kt(ctx, label);
#define PLX_BD(TM, TN)                                                                                              \
    st = run<TM, TN>(ctx, R, (int)Mp, (int)N, (const float*)P, ldp, (const float*)Q, ldq, (const float*)Zm, ldz, W, ldw, \
                     (float*)dOut, ldo, part, rpc, chunks, mask_bits, vec, split, fac)
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
