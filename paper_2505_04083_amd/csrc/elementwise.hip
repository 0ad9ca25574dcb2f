// Element-wise steps of a GCN layer (paper Eq. 2.3 activation, Eq. 2.4 its derivative) and the
// node-classification loss head (Sec. 2.1: softmax cross-entropy averaged over all nodes).
// All are streaming kernels bound by HBM bandwidth.
#include "plx_internal.h"

#include <algorithm>

namespace plx {
namespace {

typedef uint16_t bf16_t;

__device__ __forceinline__ float widen(float v) { return v; }
__device__ __forceinline__ float widen(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }
template <typename T> __device__ __forceinline__ T narrow(float f);
template <> __device__ __forceinline__ float narrow<float>(float f) { return f; }
template <> __device__ __forceinline__ bf16_t narrow<bf16_t>(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// F = max(Z, 0); 2-D indexing so padded leading dimensions are never touched
template <typename T>
__global__ __launch_bounds__(256) void k_relu(int64_t rows, int cols, const T* __restrict__ Z, int64_t ldz, T* F,
                                              int64_t ldf) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= cols) return;
    for (int64_t r = blockIdx.y; r < rows; r += gridDim.y) {
        float z = widen(Z[r * ldz + c]);
        F[r * ldf + c] = narrow<T>(z > 0.f ? z : 0.f);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void k_relu_bwd(int64_t rows, int cols, const T* Z, int64_t ldz, const T* dF,
                                                  int64_t lddf, T* dZ, int64_t lddz) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= cols) return;
    for (int64_t r = blockIdx.y; r < rows; r += gridDim.y) {
        float z = widen(Z[r * ldz + c]);
        float g = widen(dF[r * lddf + c]);
        dZ[r * lddz + c] = narrow<T>(z > 0.f ? g : 0.f);
    }
}

// bits[r][j / 32] bit j % 32 = [F[r][j] > 0]: one wavefront per 64 columns of a row, two words per ballot
template <typename T>
__global__ __launch_bounds__(256) void k_bits_from_act(int64_t rows, int cols, const T* __restrict__ F, int64_t ldf,
                                                       uint32_t* __restrict__ bits, int64_t ldbits) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + lane;
    for (int64_t r = (int64_t)blockIdx.y * 4 + wv; r < rows; r += (int64_t)gridDim.y * 4) {
        const bool pos = c < cols && widen(F[r * ldf + c]) > 0.f;
        const unsigned long long b = __ballot(pos);
        const int word = blockIdx.x * 2 + (lane >> 5);
        if ((lane & 31) == 0 && word * 32 < cols) bits[r * ldbits + word] = (uint32_t)(b >> (32 * (lane >> 5)));
    }
}

// dZ = dF where the sign bit of the forward product is set, else 0
template <typename T>
__global__ __launch_bounds__(256) void k_relu_bwd_bits(int64_t rows, int cols, const uint32_t* __restrict__ bits,
                                                       int64_t ldbits, const T* dF, int64_t lddf, T* dZ, int64_t lddz) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= cols) return;
    for (int64_t r = blockIdx.y; r < rows; r += gridDim.y) {
        const uint32_t m = bits[r * ldbits + (c >> 5)] >> (c & 31) & 1u;
        dZ[r * lddz + c] = m ? dF[r * lddf + c] : narrow<T>(0.f);
    }
}

// contiguous matrices: 4 elements per thread
template <typename T>
__global__ __launch_bounds__(256) void k_relu_flat(int64_t count, const T* __restrict__ Z, T* F) {
    int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i + 3 < count) {
        T z[4];
        if constexpr (sizeof(T) == 4) *reinterpret_cast<uint4*>(z) = *reinterpret_cast<const uint4*>(Z + i);
        else *reinterpret_cast<uint2*>(z) = *reinterpret_cast<const uint2*>(Z + i);
#pragma unroll
        for (int t = 0; t < 4; ++t) { float v = widen(z[t]); z[t] = narrow<T>(v > 0.f ? v : 0.f); }
        if constexpr (sizeof(T) == 4) *reinterpret_cast<uint4*>(F + i) = *reinterpret_cast<uint4*>(z);
        else *reinterpret_cast<uint2*>(F + i) = *reinterpret_cast<uint2*>(z);
    } else {
        for (; i < count; ++i) { float v = widen(Z[i]); F[i] = narrow<T>(v > 0.f ? v : 0.f); }
    }
}

template <typename T>
__global__ __launch_bounds__(256) void k_relu_bwd_flat(int64_t count, const T* Z, const T* dF, T* dZ) {
    int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i + 3 < count) {
        T z[4], g[4];
        if constexpr (sizeof(T) == 4) {
            *reinterpret_cast<uint4*>(z) = *reinterpret_cast<const uint4*>(Z + i);
            *reinterpret_cast<uint4*>(g) = *reinterpret_cast<const uint4*>(dF + i);
        } else {
            *reinterpret_cast<uint2*>(z) = *reinterpret_cast<const uint2*>(Z + i);
            *reinterpret_cast<uint2*>(g) = *reinterpret_cast<const uint2*>(dF + i);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) g[t] = widen(z[t]) > 0.f ? g[t] : narrow<T>(0.f);
        if constexpr (sizeof(T) == 4) *reinterpret_cast<uint4*>(dZ + i) = *reinterpret_cast<uint4*>(g);
        else *reinterpret_cast<uint2*>(dZ + i) = *reinterpret_cast<uint2*>(g);
    } else {
        for (; i < count; ++i) dZ[i] = widen(Z[i]) > 0.f ? dF[i] : narrow<T>(0.f);
    }
}

// One group of GS lanes per node (GS a power of two <= 64): lane t of the group holds classes
// t, t + GS, ... so the row is read and the gradient written with coalesced accesses; row max and
// sum of exponentials are butterfly reductions inside the group.
template <typename T, int GS, int MAXV>   // c <= GS * MAXV
__global__ __launch_bounds__(256) void k_softmax_ce(int64_t n, int c, const T* __restrict__ Z, int64_t ldz,
                                                    const int64_t* __restrict__ y, T* __restrict__ dZ, int64_t lddz,
                                                    float* __restrict__ row_loss, float inv_n) {
    const int t = threadIdx.x % GS;
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / GS;
    const bool live = i < n;
    const T* z = Z + (live ? i : 0) * ldz;
    float v[MAXV];
    float mx = -INFINITY;
#pragma unroll
    for (int q = 0; q < MAXV; ++q) {
        const int j = t + q * GS;
        v[q] = (live && j < c) ? widen(z[j]) : -INFINITY;
        mx = fmaxf(mx, v[q]);
    }
#pragma unroll
    for (int off = GS / 2; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, GS));
    float sum = 0.f;
#pragma unroll
    for (int q = 0; q < MAXV; ++q) {
        v[q] = (t + q * GS < c) ? expf(v[q] - mx) : 0.f;
        sum += v[q];
    }
#pragma unroll
    for (int off = GS / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off, GS);
    if (!live) return;
    const float inv = 1.f / sum;
    int64_t label = y[i];
    label = label < 0 ? 0 : (label >= c ? c - 1 : label);   // out-of-range labels are clamped
    T* g = dZ + i * lddz;
#pragma unroll
    for (int q = 0; q < MAXV; ++q) {
        const int j = t + q * GS;
        if (j < c) g[j] = narrow<T>((v[q] * inv - (j == label ? 1.f : 0.f)) * inv_n);
    }
    if (t == 0) row_loss[i] = -(widen(z[label]) - mx - logf(sum));
}

// fp32 rows that are 16-byte aligned: lane t of a group of GS lanes holds classes 4t .. 4t+3 as one
// 128-bit load and writes its part of the gradient as one 128-bit store (c <= 4 * GS)
template <int GS>
__global__ __launch_bounds__(256) void k_softmax_ce_v4(int64_t n, int c, const float* __restrict__ Z, int64_t ldz,
                                                       const int64_t* __restrict__ y, float* __restrict__ dZ, int64_t lddz,
                                                       float* __restrict__ row_loss, float inv_n) {
    const int t = threadIdx.x % GS, j0 = 4 * t;
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / GS;
    const bool live = i < n;
    const float* z = Z + (live ? i : 0) * ldz;
    float v[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    if (live && j0 + 3 < c) {
        const float4 q = *reinterpret_cast<const float4*>(z + j0);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    } else if (live) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (j0 + e < c) v[e] = z[j0 + e];
    }
    float mx = fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3]));
#pragma unroll
    for (int off = GS / 2; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, GS));
    float sum = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        v[e] = (j0 + e < c) ? expf(v[e] - mx) : 0.f;
        sum += v[e];
    }
#pragma unroll
    for (int off = GS / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off, GS);
    if (!live) return;
    const float inv = 1.f / sum;
    int64_t label = y[i];
    label = label < 0 ? 0 : (label >= c ? c - 1 : label);   // out-of-range labels are clamped
    float* g = dZ + i * lddz;
    float o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (v[e] * inv - (j0 + e == label ? 1.f : 0.f)) * inv_n;
    if (j0 + 3 < c) {
        *reinterpret_cast<float4*>(g + j0) = make_float4(o[0], o[1], o[2], o[3]);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (j0 + e < c) g[j0 + e] = o[e];
    }
    if (t == 0) row_loss[i] = -(z[label] - mx - logf(sum));
}

// bf16 rows that are 16-byte aligned: the same with 8 classes per lane (c <= 8 * GS)
template <int GS>
__global__ __launch_bounds__(256) void k_softmax_ce_v8(int64_t n, int c, const bf16_t* __restrict__ Z, int64_t ldz,
                                                       const int64_t* __restrict__ y, bf16_t* __restrict__ dZ, int64_t lddz,
                                                       float* __restrict__ row_loss, float inv_n) {
    const int t = threadIdx.x % GS, j0 = 8 * t;
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / GS;
    const bool live = i < n;
    const bf16_t* z = Z + (live ? i : 0) * ldz;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = -INFINITY;
    if (live && j0 + 7 < c) {
        union { uint4 raw; bf16_t e[8]; } u;
        u.raw = *reinterpret_cast<const uint4*>(z + j0);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = widen(u.e[e]);
    } else if (live) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (j0 + e < c) v[e] = widen(z[j0 + e]);
    }
    float mx = v[0];
#pragma unroll
    for (int e = 1; e < 8; ++e) mx = fmaxf(mx, v[e]);
#pragma unroll
    for (int off = GS / 2; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, GS));
    float sum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        v[e] = (j0 + e < c) ? expf(v[e] - mx) : 0.f;
        sum += v[e];
    }
#pragma unroll
    for (int off = GS / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off, GS);
    if (!live) return;
    const float inv = 1.f / sum;
    int64_t label = y[i];
    label = label < 0 ? 0 : (label >= c ? c - 1 : label);   // out-of-range labels are clamped
    bf16_t* g = dZ + i * lddz;
    union { uint4 raw; bf16_t e[8]; } o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o.e[e] = narrow<bf16_t>((v[e] * inv - (j0 + e == label ? 1.f : 0.f)) * inv_n);
    if (j0 + 7 < c) {
        *reinterpret_cast<uint4*>(g + j0) = o.raw;
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (j0 + e < c) g[j0 + e] = o.e[e];
    }
    if (t == 0) row_loss[i] = -(widen(z[label]) - mx - logf(sum));
}

// Fixed-order sum: the live slots are `stride` apart; block b adds the 2048 live slots of its range
// (8 per thread, then a tree in LDS) into the first of them.  Repeated until one slot is left.
__global__ __launch_bounds__(256) void k_sum_level(float* v, int64_t n_live, int64_t stride, float* out, float scale) {
    __shared__ float sh[256];
    const int64_t base = (int64_t)blockIdx.x * 2048;
    float s = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int64_t slot = base + threadIdx.x + 256 * q;
        if (slot < n_live) s += v[slot * stride];
    }
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) sh[threadIdx.x] += sh[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        if (out) *out = sh[0] * scale;
        else v[base * stride] = sh[0];
    }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// rows x cols elements of `bytes_per_elt` bytes each set to zero (a kernel, not a memset: memset nodes recorded
// into a HIP graph have replayed wrongly on this platform)
__global__ __launch_bounds__(256) void k_zero(int64_t rows, int64_t row_bytes, unsigned char* p, int64_t pitch_bytes) {
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= row_bytes) return;
    for (int64_t r = blockIdx.y; r < rows; r += gridDim.y) p[r * pitch_bytes + b] = 0;
}

dim3 grid2d(int64_t rows, int64_t cols) {
    unsigned gx = (unsigned)ceil_div(cols, 256);
    unsigned gy = (unsigned)std::min<int64_t>(rows, std::max<int64_t>(1, 65535));
    return dim3(gx, gy);
}

template <typename T>
plx_status relu_t(plx_ctx* ctx, int64_t rows, int64_t cols, const void* Z, int64_t ldz, void* F, int64_t ldf) {
    hipStream_t s = ctx->stream;
    char label[64];
    snprintf(label, sizeof label, "relu[R%lld,C%lld]", (long long)rows, (long long)cols);
    KernelTimer kt(ctx, label);
    if (ldz == cols && ldf == cols && aligned16(Z) && aligned16(F)) {
        int64_t count = rows * cols;
        k_relu_flat<T><<<dim3((unsigned)ceil_div(ceil_div(count, 4), 256)), 256, 0, s>>>(count, (const T*)Z, (T*)F);
    } else {
        k_relu<T><<<grid2d(rows, cols), 256, 0, s>>>(rows, (int)cols, (const T*)Z, ldz, (T*)F, ldf);
    }
    PLX_HIP(ctx, hipGetLastError());
    return PLX_OK;
}

template <typename T>
plx_status relu_bwd_t(plx_ctx* ctx, int64_t rows, int64_t cols, const void* Z, int64_t ldz, const void* dF,
                      int64_t lddf, void* dZ, int64_t lddz) {
    hipStream_t s = ctx->stream;
    char label[64];
    snprintf(label, sizeof label, "relu_bwd[R%lld,C%lld]", (long long)rows, (long long)cols);
    KernelTimer kt(ctx, label);
    if (ldz == cols && lddf == cols && lddz == cols && aligned16(Z) && aligned16(dF) && aligned16(dZ)) {
        int64_t count = rows * cols;
        k_relu_bwd_flat<T><<<dim3((unsigned)ceil_div(ceil_div(count, 4), 256)), 256, 0, s>>>(count, (const T*)Z,
                                                                                           (const T*)dF, (T*)dZ);
    } else {
        k_relu_bwd<T><<<grid2d(rows, cols), 256, 0, s>>>(rows, (int)cols, (const T*)Z, ldz, (const T*)dF, lddf, (T*)dZ, lddz);
    }
    PLX_HIP(ctx, hipGetLastError());
    return PLX_OK;
}

}  // namespace

plx_status launch_zero(plx_ctx* ctx, int64_t rows, int64_t cols, void* p, int64_t ld, size_t elt_bytes) {
    if (rows <= 0 || cols <= 0 || !p) return PLX_OK;
    const int64_t row_bytes = cols * (int64_t)elt_bytes;
    dim3 grid((unsigned)ceil_div(row_bytes, 256), (unsigned)std::min<int64_t>(rows, 65535));
    k_zero<<<grid, 256, 0, ctx->stream>>>(rows, row_bytes, static_cast<unsigned char*>(p), ld * (int64_t)elt_bytes);
    PLX_HIP(ctx, hipGetLastError());
    return PLX_OK;
}

plx_status launch_relu(plx_ctx* ctx, int64_t rows, int64_t cols, const void* Z, int64_t ldz, void* F, int64_t ldf,
                       plx_dtype dtype) {
    if (cols >= (int64_t(1) << 24)) return fail(ctx, PLX_ERR_UNSUPPORTED, "too many columns");
    return dtype == PLX_F32 ? relu_t<float>(ctx, rows, cols, Z, ldz, F, ldf) : relu_t<bf16_t>(ctx, rows, cols, Z, ldz, F, ldf);
}

plx_status launch_bits_from_act(plx_ctx* ctx, int64_t rows, int64_t cols, const void* F, int64_t ldf, uint32_t* bits,
                                int64_t ldbits, plx_dtype dtype) {
    if (cols >= (int64_t(1) << 24)) return fail(ctx, PLX_ERR_UNSUPPORTED, "too many columns");
    if (rows == 0 || cols == 0) return PLX_OK;
    char label[64];
    snprintf(label, sizeof label, "sign_bits[R%lld,C%lld]", (long long)rows, (long long)cols);
    KernelTimer kt(ctx, label);
    dim3 grid((unsigned)ceil_div(cols, 64), (unsigned)std::min<int64_t>(ceil_div(rows, 4), 65535));
    if (dtype == PLX_F32) k_bits_from_act<float><<<grid, 256, 0, ctx->stream>>>(rows, (int)cols, (const float*)F, ldf, bits, ldbits);
    else k_bits_from_act<bf16_t><<<grid, 256, 0, ctx->stream>>>(rows, (int)cols, (const bf16_t*)F, ldf, bits, ldbits);
    PLX_HIP(ctx, hipGetLastError());
    return PLX_OK;
}

plx_status launch_relu_bwd(plx_ctx* ctx, int64_t rows, int64_t cols, const void* Z, int64_t ldz, const void* dF,
                           int64_t lddf, void* dZ, int64_t lddz, plx_dtype dtype, bool mask_bits) {
    if (cols >= (int64_t(1) << 24)) return fail(ctx, PLX_ERR_UNSUPPORTED, "too many columns");
    if (mask_bits) {
        if (rows == 0 || cols == 0) return PLX_OK;
        char label[64];
        snprintf(label, sizeof label, "relu_bwd_bits[R%lld,C%lld]", (long long)rows, (long long)cols);
        KernelTimer kt(ctx, label);
        const uint32_t* b = (const uint32_t*)Z;
        if (dtype == PLX_F32)
            k_relu_bwd_bits<float><<<grid2d(rows, cols), 256, 0, ctx->stream>>>(rows, (int)cols, b, ldz, (const float*)dF, lddf, (float*)dZ, lddz);
        else
            k_relu_bwd_bits<bf16_t><<<grid2d(rows, cols), 256, 0, ctx->stream>>>(rows, (int)cols, b, ldz, (const bf16_t*)dF, lddf, (bf16_t*)dZ, lddz);
        PLX_HIP(ctx, hipGetLastError());
        return PLX_OK;
    }
    return dtype == PLX_F32 ? relu_bwd_t<float>(ctx, rows, cols, Z, ldz, dF, lddf, dZ, lddz)
                            : relu_bwd_t<bf16_t>(ctx, rows, cols, Z, ldz, dF, lddf, dZ, lddz);
}

plx_status launch_softmax_ce(plx_ctx* ctx, int64_t n, int64_t c, const void* Z, int64_t ldz, const int64_t* y, void* dZ,
                             int64_t lddz, float* row_loss, float* loss, plx_dtype dtype) {
    hipStream_t s = ctx->stream;
    if (n == 0) {
        return launch_zero(ctx, 1, 1, loss, 1, sizeof(float));
    }
    const float inv_n = (float)(1.0 / (double)n);
    char label[64];
    snprintf(label, sizeof label, "softmax_ce[R%lld,C%lld]", (long long)n, (long long)c);
    KernelTimer kt(ctx, label);
    if (dtype == PLX_F32 && c <= 256 && ldz % 4 == 0 && lddz % 4 == 0 && aligned16(Z) && aligned16(dZ)) {
        const int q = (int)ceil_div(c, 4);
        const int g4 = q <= 4 ? 4 : (q <= 8 ? 8 : (q <= 16 ? 16 : (q <= 32 ? 32 : 64)));
        dim3 grid4((unsigned)ceil_div(n * g4, 256));
#define PLX_SM4(GSV) k_softmax_ce_v4<GSV><<<grid4, 256, 0, s>>>(n, (int)c, (const float*)Z, ldz, y, (float*)dZ, lddz, row_loss, inv_n)
        if (g4 == 4) PLX_SM4(4); else if (g4 == 8) PLX_SM4(8); else if (g4 == 16) PLX_SM4(16); else if (g4 == 32) PLX_SM4(32); else PLX_SM4(64);
#undef PLX_SM4
    } else if (dtype == PLX_BF16 && c <= 512 && ldz % 8 == 0 && lddz % 8 == 0 && aligned16(Z) && aligned16(dZ)) {
        const int q = (int)ceil_div(c, 8);
        const int g8 = q <= 2 ? 2 : (q <= 4 ? 4 : (q <= 8 ? 8 : (q <= 16 ? 16 : (q <= 32 ? 32 : 64))));
        dim3 grid8((unsigned)ceil_div(n * g8, 256));
#define PLX_SM8(GSV) k_softmax_ce_v8<GSV><<<grid8, 256, 0, s>>>(n, (int)c, (const bf16_t*)Z, ldz, y, (bf16_t*)dZ, lddz, row_loss, inv_n)
        if (g8 == 2) PLX_SM8(2); else if (g8 == 4) PLX_SM8(4); else if (g8 == 8) PLX_SM8(8); else if (g8 == 16) PLX_SM8(16);
        else if (g8 == 32) PLX_SM8(32); else PLX_SM8(64);
#undef PLX_SM8
    } else {
    const int gs = c <= 32 ? 8 : (c <= 64 ? 16 : (c <= 128 ? 32 : 64));
    dim3 grid((unsigned)ceil_div(n * gs, 256));
#define PLX_SM(TT, GSV) \
    k_softmax_ce<TT, GSV, (GSV == 64 ? 16 : 4)><<<grid, 256, 0, s>>>(n, (int)c, (const TT*)Z, ldz, y, (TT*)dZ, lddz, row_loss, inv_n)
    if (dtype == PLX_F32) {
        if (gs == 8) PLX_SM(float, 8); else if (gs == 16) PLX_SM(float, 16); else if (gs == 32) PLX_SM(float, 32); else PLX_SM(float, 64);
    } else {
        if (gs == 8) PLX_SM(bf16_t, 8); else if (gs == 16) PLX_SM(bf16_t, 16); else if (gs == 32) PLX_SM(bf16_t, 32); else PLX_SM(bf16_t, 64);
    }
#undef PLX_SM
    }
    if (loss) {
        int64_t live = n, stride = 1;
        while (true) {
            const int64_t groups = ceil_div(live, 2048);
            const bool last = groups == 1;
            k_sum_level<<<dim3((unsigned)groups), 256, 0, s>>>(row_loss, live, stride, last ? loss : nullptr, inv_n);
            if (last) break;
            live = groups;
            stride *= 2048;
        }
    }
    PLX_HIP(ctx, hipGetLastError());
    return PLX_OK;
}

}  // namespace plx
