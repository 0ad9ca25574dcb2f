// Device-side helpers shared by the kernels that feed bf16 matrix instructions: the 16-byte fragment
// union, hardware rounding to bf16, and the two ways an operand fragment is read from a row-major
// LDS tile (8 consecutive k of a row; 8 consecutive rows of a column through the transpose read).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace plx {
namespace {

typedef uint16_t bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4_t;
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define PLX_LDS __attribute__((address_space(3)))

union Frag {
    uint4 u;
    u32x4 x;
    bf16x8 v;
    bf16x4_t h[2];
    bf16_t e[8];
};

__device__ __forceinline__ bf16_t f32_to_bf16(float f) {   // round to nearest even: one v_cvt_pk_bf16_f32
    return __builtin_bit_cast(bf16_t, (__bf16)f);
}
__device__ __forceinline__ bool bf16_positive(bf16_t z) { return (z & 0x8000u) == 0 && (z & 0x7fffu) != 0 && (z & 0x7fffu) <= 0x7f80u; }

// 8 consecutive bf16 of one row (16 bytes)
__device__ __forceinline__ bf16x8 frag_contig(const bf16_t* p) {
    Frag f;
    f.u = *reinterpret_cast<const uint4*>(p);
    return f.v;
}

// Column fragment of a row-major LDS tile for a 32x32x16 operand: lane l receives rows
// k0 + 8*(l/32) .. +7 of column c0 + l%32.  Two transpose reads of 4 rows each.
__device__ __forceinline__ bf16x8 frag_column(const bf16_t* tile, int pitch, int k0, int c0, int lane) {
    const int L = lane & 15, half = (lane >> 4) & 1, lh = lane >> 5;
    const bf16_t* p = tile + (k0 + 8 * lh + (L >> 2)) * pitch + c0 + 16 * half + 4 * (L & 3);
    Frag f;
    f.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((PLX_LDS bf16x4_t*)(p));
    f.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((PLX_LDS bf16x4_t*)(p + 4 * pitch));
    return f.v;
}

// ---- fp32 products through the bf16 matrix instructions ------------------------------------------------
// split3: v = pl[0] + pl[1] + pl[2] element-wise (exact for finite v: 8 + 8 + 8 significand bits); four elements
// per call, returned as packed pairs.  The leading part must not overflow: rounding a finite element within 0.4 % of
// the largest fp32 value to nearest would give infinity, and infinity minus infinity would turn the other parts into
// NaN.  Row tiles (kWeights == false, the per-tile hot path) therefore take the leading part by TRUNCATION -- one byte
// permute per pair, the cost of the conversion it replaces; what is left has the sign of the element and fewer than
// 16 significant bits, so the two nearest-even parts that follow still end exactly.  Weight slices (kWeights == true,
// split once per kernel) round all three parts to nearest even and fall back to the truncated leading part only where
// the rounded one is infinite and the element is not: with them |b2| <= 2^-9 |b|, |b3| <= 2^-17 |b|, and with the row
// tiles |a2| < 2^-7 |a|, |a3| <= 2^-16 |a|.  An infinite or NaN element makes its parts, and every sum it enters, NaN.
// PLX_X3_16 / PLX_X3_32: acc += a b over the six products that matter (a1 b1, a1 b2, a2 b1, a2 b2, a1 b3, a3 b1);
// the three dropped ones are below 2^-24 |a b| each, i.e. below the rounding of an fp32 product.
template <bool kWeights = false>
__device__ __forceinline__ void split3(const float4& v, uint2 (&pl)[3]) {
    typedef float f2 __attribute__((ext_vector_type(2)));
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    float x[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int p = 0; p < 3; ++p) {
        uint32_t wl, wh;
        if (p == 0) {
            // upper halves of two fp32 words packed into one: low half from the first element
            const uint32_t tl = __builtin_amdgcn_perm(__float_as_uint(x[1]), __float_as_uint(x[0]), 0x07060302u);
            const uint32_t th = __builtin_amdgcn_perm(__float_as_uint(x[3]), __float_as_uint(x[2]), 0x07060302u);
            if (kWeights) {
                wl = __builtin_bit_cast(uint32_t, __builtin_convertvector((f2){x[0], x[1]}, b2));
                wh = __builtin_bit_cast(uint32_t, __builtin_convertvector((f2){x[2], x[3]}, b2));
                auto fix = [](uint32_t r, uint32_t t) {      // per half: rounded part infinite, truncated part not -> truncated
                    const uint32_t lo = ((r & 0x7fffu) == 0x7f80u && (t & 0x7fffu) != 0x7f80u) ? (t & 0xffffu) : (r & 0xffffu);
                    const uint32_t hi = ((r & 0x7fff0000u) == 0x7f800000u && (t & 0x7fff0000u) != 0x7f800000u) ? (t & 0xffff0000u)
                                                                                                               : (r & 0xffff0000u);
                    return lo | hi;
                };
                wl = fix(wl, tl); wh = fix(wh, th);
            } else {
                wl = tl; wh = th;
            }
        } else {
            wl = __builtin_bit_cast(uint32_t, __builtin_convertvector((f2){x[0], x[1]}, b2));
            wh = __builtin_bit_cast(uint32_t, __builtin_convertvector((f2){x[2], x[3]}, b2));
        }
        pl[p] = make_uint2(wl, wh);
        if (p < 2) {                   // exact: the part shares the leading bits of x
            x[0] -= __uint_as_float(wl << 16); x[1] -= __uint_as_float(wl & 0xffff0000u);
            x[2] -= __uint_as_float(wh << 16); x[3] -= __uint_as_float(wh & 0xffff0000u);
        }
    }
}
// acc += a b over the six kept products, smallest first
#define PLX_X3_16(acc, a, b)                                                                   \
    do {                                                                                       \
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[2], b[0], acc, 0, 0, 0);               \
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[0], b[2], acc, 0, 0, 0);               \
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[1], b[1], acc, 0, 0, 0);               \
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[1], b[0], acc, 0, 0, 0);               \
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[0], b[1], acc, 0, 0, 0);               \
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[0], b[0], acc, 0, 0, 0);               \
    } while (0)
#define PLX_X3_32(acc, a, b)                                                                   \
    do {                                                                                       \
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2], b[0], acc, 0, 0, 0);               \
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[2], acc, 0, 0, 0);               \
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[1], acc, 0, 0, 0);               \
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[0], acc, 0, 0, 0);               \
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[1], acc, 0, 0, 0);               \
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[0], acc, 0, 0, 0);               \
    } while (0)

}  // namespace
}  // namespace plx
