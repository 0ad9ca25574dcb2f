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
// split3: v = pl[0] + pl[1] + pl[2] element-wise, each part a bf16 rounded to nearest even from what
// the earlier parts leave (exact for finite v: 8 + 8 + 8 significand bits); four elements per call,
// returned as packed pairs.  PLX_X3_16 / PLX_X3_32: acc += a b over the six products that matter
// (a1 b1, a1 b2, a2 b1, a2 b2, a1 b3, a3 b1: everything down to 2^-23 |a b|), smallest first.
__device__ __forceinline__ void split3(const float4& v, uint2 (&pl)[3]) {
    typedef float f2 __attribute__((ext_vector_type(2)));
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    float x[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int p = 0; p < 3; ++p) {
        const uint32_t wl = __builtin_bit_cast(uint32_t, __builtin_convertvector((f2){x[0], x[1]}, b2));
        const uint32_t wh = __builtin_bit_cast(uint32_t, __builtin_convertvector((f2){x[2], x[3]}, b2));
        pl[p] = make_uint2(wl, wh);
        if (p < 2) {                   // exact: the rounded part shares the leading bits of x
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
