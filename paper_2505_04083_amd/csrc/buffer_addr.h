// Device-side helpers shared by the dense kernels: buffer addressing and a one-instruction ReLU.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace plx {

// max(v, 0) in one vector instruction (the compiler's own form adds a canonicalising second one)
__device__ __forceinline__ float relu0(float v) {
    float o;
    asm("v_max_f32 %0, 0, %1" : "=v"(o) : "v"(v));
    return o;
}

// Buffer addressing: a 128-bit descriptor in scalar registers (base, byte count), a 32-bit byte offset
// per lane and a scalar byte offset.  Vector instructions take issue cycles from the matrix pipe
// (measured: 3-4 cycles per wave-wide instruction, no overlap), so the kernels below keep every
// per-tile and per-row address step on the scalar unit: the lane offsets are computed once per
// kernel.  Loads beyond the byte count return 0, which also serves the rows past the end of a
// matrix and the padded columns.
constexpr int kRawBuffer = 0x00020000;            // descriptor word 3 of an untyped buffer on gfx9-family devices
constexpr uint32_t kOutOfRange = 0x80000000u;     // a lane offset no descriptor below reaches
__device__ __forceinline__ __amdgpu_buffer_rsrc_t buffer_of(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, kRawBuffer);
}
__device__ __forceinline__ float4 buffer_load4(__amdgpu_buffer_rsrc_t r, uint32_t lane_off) {
    return __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_off, 0, 0));
}
__device__ __forceinline__ uint32_t buffer_load1(__amdgpu_buffer_rsrc_t r, uint32_t lane_off) {
    return __builtin_amdgcn_raw_buffer_load_b32(r, (int)lane_off, 0, 0);
}
// non-temporal: results are not read again by this kernel
__device__ __forceinline__ void buffer_store_nt(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t row_off, float v) {
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, (int)lane_off, (int)row_off, 2);
}
// plain store (the result is read again soon, by the sparse product that follows); stores beyond the byte count are dropped
__device__ __forceinline__ void buffer_store(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t row_off, float v) {
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, (int)lane_off, (int)row_off, 0);
}
// A zero the optimiser cannot see through: row offsets that start from it are recomputed per tile with
// scalar additions instead of being hoisted out of the tile loop into (spilled) scalar registers.
__device__ __forceinline__ uint32_t opaque_zero() {
    uint32_t z = 0;
    asm volatile("" : "+s"(z));
    return z;
}

}  // namespace plx
