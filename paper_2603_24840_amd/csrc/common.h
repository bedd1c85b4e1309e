// Shared host/device helpers for the ARRoL HIP library (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include <tuple>
#include <type_traits>
#include <utility>
#include "arrol.h"

#define ARROL_WAVE 64

// 16-byte native vector (the nontemporal builtins need a native vector, not HIP's uint4 class)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Kernel launches go through arrol_launch(), which keeps the runtime's OWN return value of each launch
// (hipLaunchKernel) in a per-thread slot: an error some earlier, unrelated HIP call of the caller left in
// the thread's sticky error state is neither reported as a failure of this library nor cleared from the
// caller's view.  arrol_launch_failed() peeks at the slot between the launches of one entry point;
// arrol_launch_status() turns it into the entry point's return code and empties it.
inline hipError_t& arrol_launch_error_slot() {
    static thread_local hipError_t err = hipSuccess;
    return err;
}
template <class Tuple, size_t... I>
static inline hipError_t arrol_launch_packed(const void* fn, dim3 grid, dim3 block, size_t lds, hipStream_t st,
                                             Tuple& vals, std::index_sequence<I...>) {
    void* ptrs[] = {static_cast<void*>(&std::get<I>(vals))..., nullptr};
    return hipLaunchKernel(fn, grid, block, ptrs, lds, st);
}
template <class... KArgs, class... Args>
static inline void arrol_launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t st,
                                Args&&... args) {
    static_assert(sizeof...(KArgs) == sizeof...(Args), "one argument per kernel parameter");
    hipError_t& slot = arrol_launch_error_slot();
    if (slot != hipSuccess) return;   // an earlier launch of this entry point failed: enqueue nothing more
    std::tuple<std::remove_cv_t<KArgs>...> vals(static_cast<KArgs>(args)...);
    slot = arrol_launch_packed(reinterpret_cast<const void*>(kernel), grid, block, lds, st, vals,
                               std::index_sequence_for<KArgs...>{});
}
static inline bool arrol_launch_failed() { return arrol_launch_error_slot() != hipSuccess; }
static inline int arrol_launch_status() {
    hipError_t& slot = arrol_launch_error_slot();
    const bool ok = slot == hipSuccess;
    slot = hipSuccess;
    return ok ? ARROL_OK : ARROL_EHIP;
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
