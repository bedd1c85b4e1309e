// Measurement aid, not a stage of the pruning path: the rate at which this card's matrix cores run bf16 MFMAs
// from registers alone - no LDS, no global loads, no epilogue, two wavefronts per SIMD as in the log-prob kernel -
// on operand values the caller supplies.  On operands that toggle (the workloads' N(0,1) data) the part's power
// control lowers the shader clock, on all-zero operands it does not: the two rates bracket what any kernel built
// from these instructions can reach on the same card, and the benchmark prints them next to the log-prob kernel's.
#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kProbeThreads = 512;   // 8 wavefronts = 2 per SIMD
constexpr int kProbeFragsA = 8, kProbeFragsB = 4;

// fragment f of wavefront w: 64 lanes x 16 bytes, taken round-robin from the operand buffer
__device__ inline bf16x8 probe_fragment(const bf16x8* __restrict__ src, int64_t n_frag, int64_t w, int f, int per_wave,
                                        int lane) {
    const int64_t idx = (w * per_wave + f) % n_frag;
    return src[idx * ARROL_WAVE + lane];
}

// SHAPE 16: v_mfma_f32_16x16x32_bf16, 32 accumulators of 4 registers (the log-prob kernel's 8 x 4 tile of blocks);
// SHAPE 32: v_mfma_f32_32x32x16_bf16, 8 accumulators of 16 registers, two K halves each.  Both forms do the same
// 524,288 flop per wavefront and iteration (32 instructions of 2*16*16*32, resp. 16 of 2*32*32*16).
template <int SHAPE>
__global__ __launch_bounds__(kProbeThreads) void mfma_rate_kernel(const bf16x8* __restrict__ a_src, int64_t n_frag_a,
                                                                  const bf16x8* __restrict__ b_src, int64_t n_frag_b,
                                                                  int iters, float* __restrict__ sink) {
    const int lane = threadIdx.x & (ARROL_WAVE - 1);
    const int64_t w = static_cast<int64_t>(blockIdx.x) * (kProbeThreads / ARROL_WAVE) + threadIdx.x / ARROL_WAVE;
    bf16x8 a[kProbeFragsA], b[kProbeFragsB];
#pragma unroll
    for (int f = 0; f < kProbeFragsA; ++f) a[f] = probe_fragment(a_src, n_frag_a, w, f, kProbeFragsA, lane);
#pragma unroll
    for (int f = 0; f < kProbeFragsB; ++f) b[f] = probe_fragment(b_src, n_frag_b, w, f, kProbeFragsB, lane);
    float s = 0.f;
    if (SHAPE == 16) {
        f32x4 acc[32];
#pragma unroll
        for (int x = 0; x < 32; ++x) acc[x] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int x = 0; x < 32; ++x)
                acc[x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[x >> 2], b[x & 3], acc[x], 0, 0, 0);
        }
#pragma unroll
        for (int x = 0; x < 32; ++x) s += (acc[x][0] + acc[x][1]) + (acc[x][2] + acc[x][3]);
    } else {
        f32x16 acc[8];
#pragma unroll
        for (int x = 0; x < 8; ++x)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[x][v] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int x = 0; x < 16; ++x) {
                const int blk = x & 7, half = x >> 3;
                acc[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(blk >> 1) + 4 * half], b[(blk & 1) + 2 * half],
                                                                   acc[blk], 0, 0, 0);
            }
        }
#pragma unroll
        for (int x = 0; x < 8; ++x)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += acc[x][v];
    }
    sink[static_cast<int64_t>(blockIdx.x) * kProbeThreads + threadIdx.x] = s;
}

}  // namespace

extern "C" int arrol_probe_mfma_rate(const void* a_bf16, int64_t n_a, const void* b_bf16, int64_t n_b, int32_t shape,
                                     int32_t n_workgroups, int32_t iters, float* sink, double* flop_out,
                                     void* stream) {
    if (!a_bf16 || !b_bf16 || !sink) return ARROL_EINVAL;
    if (shape != 16 && shape != 32) return ARROL_EINVAL;
    if (n_workgroups < 1 || n_workgroups > 65536 || iters < 0) return ARROL_EINVAL;
    // whole fragments only: 64 lanes x 8 bf16 values
    if (n_a < ARROL_WAVE * 8 || n_b < ARROL_WAVE * 8 || n_a % (ARROL_WAVE * 8) || n_b % (ARROL_WAVE * 8)) return ARROL_EINVAL;
    if ((reinterpret_cast<uintptr_t>(a_bf16) | reinterpret_cast<uintptr_t>(b_bf16)) & 15) return ARROL_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bf16x8* a = static_cast<const bf16x8*>(a_bf16);
    const bf16x8* b = static_cast<const bf16x8*>(b_bf16);
    const int64_t fa = n_a / (ARROL_WAVE * 8), fb = n_b / (ARROL_WAVE * 8);
    if (shape == 16)
        arrol_launch(mfma_rate_kernel<16>, dim3(n_workgroups), dim3(kProbeThreads), 0, st, a, fa, b, fb, iters, sink);
    else
        arrol_launch(mfma_rate_kernel<32>, dim3(n_workgroups), dim3(kProbeThreads), 0, st, a, fa, b, fb, iters, sink);
    if (flop_out)   // host scalar: 32 instructions of 2*16*16*32 flop (16 of 2*32*32*16) per wavefront and iteration
        *flop_out = 2.0 * 16 * 16 * 32 * 32.0 * iters * (kProbeThreads / ARROL_WAVE) * n_workgroups;
    return arrol_launch_status();
}
