// arrol_score: quality head (one linear layer) on checkpoint hidden states, then sigmoid
// (Sec. 4.2 "Quality Score Prediction"; App. A.4 score normalisation).
// HBM-streaming kernel: one wavefront per row, 16-byte loads, the head's weights staged
// once per workgroup in LDS, fp32 accumulation, butterfly reduction across the wave.
#include "common.h"

namespace {

constexpr int kScoreThreads = 512;
constexpr int kScoreWaves = kScoreThreads / ARROL_WAVE;
constexpr int kScoreUnroll = 4;          // 16-byte loads per lane in flight
constexpr int kScoreLdsFloats = 16384;  // weights up to d = 16384 live in LDS (64 KiB)

template <bool W_IN_LDS>
__global__ __launch_bounds__(kScoreThreads) void score_kernel(
    const u32x4* __restrict__ hidden, int64_t row_stride_vec, const int64_t* __restrict__ row_index,
    const float* __restrict__ w, float bias, int n_rows, int d_vec,
    float* __restrict__ score_out, float* __restrict__ prob_out) {
    extern __shared__ float w_lds[];  // d floats when W_IN_LDS, else empty
    if (W_IN_LDS) {
        for (int i = threadIdx.x; i < d_vec * 8; i += kScoreThreads) w_lds[i] = w[i];
        __syncthreads();
    }
    const int lane = threadIdx.x & (ARROL_WAVE - 1);
    const int wave = threadIdx.x / ARROL_WAVE;
    const int wave_stride = gridDim.x * kScoreWaves;
    for (int row = blockIdx.x * kScoreWaves + wave; row < n_rows; row += wave_stride) {
        const int64_t src_row = row_index ? row_index[row] : row;
        const u32x4* p = hidden + src_row * row_stride_vec;
        float acc0 = 0.f, acc1 = 0.f;
        for (int v0 = 0; v0 < d_vec; v0 += kScoreUnroll * ARROL_WAVE) {
            u32x4 x[kScoreUnroll];
#pragma unroll
            for (int u = 0; u < kScoreUnroll; ++u) {
                const int v = v0 + u * ARROL_WAVE + lane;
                x[u] = v < d_vec ? __builtin_nontemporal_load(p + v) : u32x4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int u = 0; u < kScoreUnroll; ++u) {
                const int v = v0 + u * ARROL_WAVE + lane;
                if (v < d_vec) {
                    float4 wa, wb;
                    if (W_IN_LDS) {
                        wa = *reinterpret_cast<const float4*>(w_lds + v * 8);
                        wb = *reinterpret_cast<const float4*>(w_lds + v * 8 + 4);
                    } else {
                        wa = *reinterpret_cast<const float4*>(w + v * 8);
                        wb = *reinterpret_cast<const float4*>(w + v * 8 + 4);
                    }
                    acc0 = fmaf(bf16_lo(x[u].x), wa.x, acc0);
                    acc1 = fmaf(bf16_hi(x[u].x), wa.y, acc1);
                    acc0 = fmaf(bf16_lo(x[u].y), wa.z, acc0);
                    acc1 = fmaf(bf16_hi(x[u].y), wa.w, acc1);
                    acc0 = fmaf(bf16_lo(x[u].z), wb.x, acc0);
                    acc1 = fmaf(bf16_hi(x[u].z), wb.y, acc1);
                    acc0 = fmaf(bf16_lo(x[u].w), wb.z, acc0);
                    acc1 = fmaf(bf16_hi(x[u].w), wb.w, acc1);
                }
            }
        }
        const float s = wave_sum_f32(acc0 + acc1) + bias;
        if (lane == 0) {
            float q;
            if (s >= 0.f) {
                q = 1.f / (1.f + expf(-s));
            } else {
                const float e = expf(s);
                q = e / (1.f + e);
            }
            if (score_out) score_out[row] = s;
            prob_out[row] = q;
        }
    }
}

}  // namespace

extern "C" int arrol_score(const void* hidden, int64_t row_stride_elems, const int64_t* row_index,
                           const float* w, float bias, int32_t n_rows, int32_t d,
                           float* score_out, float* prob_out, void* stream) {
    if (n_rows < 0 || d < 8 || (d & 7) || row_stride_elems < d || (row_stride_elems & 7)) return ARROL_EINVAL;
    if (n_rows == 0) return ARROL_OK;
    if (!hidden || !w || !prob_out || !arrol_aligned16(hidden) || !arrol_aligned16(w)) return ARROL_EINVAL;
    const int blocks_needed = (n_rows + kScoreWaves - 1) / kScoreWaves;
    const int grid = blocks_needed < 256 * 8 ? blocks_needed : 256 * 8;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (d <= kScoreLdsFloats) {
        hipLaunchKernelGGL(score_kernel<true>, dim3(grid), dim3(kScoreThreads), sizeof(float) * d, st,
                           static_cast<const u32x4*>(hidden), row_stride_elems / 8, row_index, w, bias,
                           n_rows, d / 8, score_out, prob_out);
    } else {
        hipLaunchKernelGGL(score_kernel<false>, dim3(grid), dim3(kScoreThreads), 0, st,
                           static_cast<const u32x4*>(hidden), row_stride_elems / 8, row_index, w, bias,
                           n_rows, d / 8, score_out, prob_out);
    }
    return arrol_launch_status();
}
