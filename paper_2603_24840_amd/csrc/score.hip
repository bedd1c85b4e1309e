// arrol_score: quality head (one linear layer) on checkpoint hidden states, then sigmoid
// (Sec. 4.2 "Quality Score Prediction"; App. A.4 score normalisation).
// HBM-streaming kernel: one wavefront per row, 16-byte non-temporal loads, fp32 accumulation, butterfly
// reduction across the wave.  Up to d = 4096 each lane keeps its slice of the head's weights in registers
// (the LDS reads of the weights, not HBM, were what bounded the kernel that staged them in LDS: 4.5 TB/s
// against 6.0-6.4 TB/s); beyond that the weights are staged in LDS, and beyond 16384 read from memory.
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

// Register variant (d <= 64*8*CH): lane l owns the 16-byte chunks c*64 + l (c < CH) of every row it sees, so
// its slice of the head's weights sits in registers for the whole kernel and a row is CH loads in flight,
// 8*CH FMAs and one butterfly.
template <int CH>
__global__ __launch_bounds__(kScoreThreads) void score_reg_kernel(
    const u32x4* __restrict__ hidden, int64_t row_stride_vec, const int64_t* __restrict__ row_index,
    const float* __restrict__ w, float bias, int n_rows, int d_vec,
    float* __restrict__ score_out, float* __restrict__ prob_out) {
    const int lane = threadIdx.x & (ARROL_WAVE - 1);
    const int wave = threadIdx.x / ARROL_WAVE;
    float4 wa[CH], wb[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int v = c * ARROL_WAVE + lane;
        wa[c] = v < d_vec ? *reinterpret_cast<const float4*>(w + v * 8) : make_float4(0.f, 0.f, 0.f, 0.f);
        wb[c] = v < d_vec ? *reinterpret_cast<const float4*>(w + v * 8 + 4) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    const int wave_stride = gridDim.x * kScoreWaves;
    for (int row = blockIdx.x * kScoreWaves + wave; row < n_rows; row += wave_stride) {
        const int64_t src_row = row_index ? row_index[row] : row;
        const u32x4* p = hidden + src_row * row_stride_vec;
        u32x4 x[CH];
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int v = c * ARROL_WAVE + lane;
            x[c] = v < d_vec ? __builtin_nontemporal_load(p + v) : u32x4{0u, 0u, 0u, 0u};
        }
        float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            acc0 = fmaf(bf16_lo(x[c].x), wa[c].x, acc0);
            acc1 = fmaf(bf16_hi(x[c].x), wa[c].y, acc1);
            acc2 = fmaf(bf16_lo(x[c].y), wa[c].z, acc2);
            acc3 = fmaf(bf16_hi(x[c].y), wa[c].w, acc3);
            acc0 = fmaf(bf16_lo(x[c].z), wb[c].x, acc0);
            acc1 = fmaf(bf16_hi(x[c].z), wb[c].y, acc1);
            acc2 = fmaf(bf16_lo(x[c].w), wb[c].z, acc2);
            acc3 = fmaf(bf16_hi(x[c].w), wb[c].w, acc3);
        }
        const float s = wave_sum_f32((acc0 + acc1) + (acc2 + acc3)) + bias;
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
    const int chunks = (d / 8 + ARROL_WAVE - 1) / ARROL_WAVE;
    if (chunks <= 8) {
        const u32x4* h = static_cast<const u32x4*>(hidden);
        const int64_t rs = row_stride_elems / 8;
#define ARROL_SCORE_REG(CH) arrol_launch(score_reg_kernel<CH>, dim3(grid), dim3(kScoreThreads), 0, st, h, rs, row_index, w, bias, n_rows, d / 8, score_out, prob_out)
        if (chunks <= 1) ARROL_SCORE_REG(1);
        else if (chunks <= 2) ARROL_SCORE_REG(2);
        else if (chunks <= 4) ARROL_SCORE_REG(4);
        else ARROL_SCORE_REG(8);
#undef ARROL_SCORE_REG
    } else if (d <= kScoreLdsFloats) {
        arrol_launch(score_kernel<true>, dim3(grid), dim3(kScoreThreads), sizeof(float) * d, st,
                           static_cast<const u32x4*>(hidden), row_stride_elems / 8, row_index, w, bias,
                           n_rows, d / 8, score_out, prob_out);
    } else {
        arrol_launch(score_kernel<false>, dim3(grid), dim3(kScoreThreads), 0, st,
                           static_cast<const u32x4*>(hidden), row_stride_elems / 8, row_index, w, bias,
                           n_rows, d / 8, score_out, prob_out);
    }
    return arrol_launch_status();
}
