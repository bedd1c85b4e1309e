// Shared host/device helpers for the ARRoL HIP library (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include "arrol.h"

#define ARROL_WAVE 64

// 16-byte native vector (the nontemporal builtins need a native vector, not HIP's uint4 class)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

static inline int arrol_launch_status() {
    return hipGetLastError() == hipSuccess ? ARROL_OK : ARROL_EHIP;
}

// Raises a kernel's dynamic-LDS limit once per device (function attributes are per device); `bytes` is the
// most the kernel is ever launched with.  Safe to call from several host threads.
typedef std::atomic<bool> arrol_device_flags[64];
template <class K>
static inline bool arrol_allow_lds(K kernel, int bytes, arrol_device_flags& done) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
    if (done[dev].load(std::memory_order_acquire)) return true;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
        return false;
    done[dev].store(true, std::memory_order_release);
    return true;
}

static inline bool arrol_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// 64-bit lane exchange built from two 32-bit shuffles.
__device__ __forceinline__ int64_t shfl_xor_i64(int64_t v, int mask) {
    int lo = __shfl_xor(static_cast<int>(v & 0xffffffffll), mask, ARROL_WAVE);
    int hi = __shfl_xor(static_cast<int>(v >> 32), mask, ARROL_WAVE);
    return (static_cast<int64_t>(hi) << 32) | static_cast<uint32_t>(lo);
}
__device__ __forceinline__ int64_t shfl_i64(int64_t v, int src) {
    int lo = __shfl(static_cast<int>(v & 0xffffffffll), src, ARROL_WAVE);
    int hi = __shfl(static_cast<int>(v >> 32), src, ARROL_WAVE);
    return (static_cast<int64_t>(hi) << 32) | static_cast<uint32_t>(lo);
}
__device__ __forceinline__ int64_t wave_sum_i64(int64_t v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += shfl_xor_i64(v, m);
    return v;
}
__device__ __forceinline__ int64_t wave_min_i64(int64_t v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) { int64_t o = shfl_xor_i64(v, m); v = o < v ? o : v; }
    return v;
}
__device__ __forceinline__ int64_t wave_max_i64(int64_t v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) { int64_t o = shfl_xor_i64(v, m); v = o > v ? o : v; }
    return v;
}
__device__ __forceinline__ float wave_sum_f32(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, ARROL_WAVE);
    return v;
}
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }
// fp32 -> bf16, round to nearest even (NaN stays a quiet NaN)
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

// out[c] = scale * sum_p partial[p*stride + c] for c < width, partials added in index order within each of
// eight interleaved groups and the groups in order: bit-reproducible.  n_partials == 0 writes zeros.
// Launch with (width + 31) / 32 workgroups of 256.
template <int kUnused = 0>
__global__ __launch_bounds__(256) void reduce_rows_f32_kernel(const float* __restrict__ partial, int n_partials,
                                                              int64_t stride, int64_t width, float scale,
                                                              float* __restrict__ out) {
    __shared__ float red[8][32];
    const int cx = threadIdx.x & 31, ry = threadIdx.x >> 5;
    const int64_t col = static_cast<int64_t>(blockIdx.x) * 32 + cx;
    float s = 0.f;
    if (col < width)
        for (int p = ry; p < n_partials; p += 8) s += partial[static_cast<int64_t>(p) * stride + col];
    red[ry][cx] = s;
    __syncthreads();
    if (ry == 0 && col < width) {
        float t = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) t += red[k][cx];
        out[col] = t * scale;
    }
}
