// arrol_score_mlp: quality head as a 2-layer MLP (Sec. 4.2: the rollout quality head "can be a simple
// 2-layer MLP"), followed by the sigmoid normalisation (App. A.4):
//     a = relu(W1 h + b1),  s = <w2, a> + b2,  q = sigmoid(s)
// One fused kernel: bf16 MFMA for W1 h (transposed, A^T = W1 H^T, so that a lane's accumulator values
// belong to one rollout and the reduction over hidden units is lane-local), bias + ReLU + the dot with w2
// on the accumulators in registers; the [N, m] activations never reach memory.
// Tile: 256 hidden units x 128 rollouts per workgroup pass, 4 wavefronts, each 2 x (32 units) x 128
// rollouts; K chunks of 64 staged global -> registers -> LDS (two stages, XOR-swizzled 16-byte chunks).
#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int BU = 256;   // hidden units per pass
constexpr int BR = 128;   // rollouts per workgroup
constexpr int BK = 64;
constexpr int TU = 2;     // 32-unit blocks per wave (unit rows c*128 + wave*32 + ...)
constexpr int TR = 4;     // 32-rollout blocks per wave
constexpr int kStageBytes = (BU + BR) * BK * 2;
constexpr int kLdsBytes = 2 * kStageBytes;
constexpr int kPassA = BU * (BK / 8) / kThreads;   // 16-byte loads per thread for the W1 tile
constexpr int kPassB = BR * (BK / 8) / kThreads;

__device__ __forceinline__ int chunk_offset(int r, int c) { return r * 128 + ((c ^ ((r >> 1) & 7)) << 4); }

struct MlpArgs {
    const uint16_t* hidden; int64_t row_stride; const int64_t* row_index;
    const uint16_t* w1; const float* b1; const float* w2; float b2;
    int n_rows, d, m;
    float* score_out; float* prob_out;
};

__global__ __launch_bounds__(kThreads) void score_mlp_kernel(MlpArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l31 = lane & 31, lh = lane >> 5;
    const int row0 = blockIdx.x * BR;

    // staging geometry: thread -> (tile row tid/8 (+32 per pass), 16-byte chunk tid%8)
    const int ld_c = tid & 7, ld_r = tid >> 3;
    const int ld_lds = chunk_offset(ld_r, ld_c);
    const uint16_t* h_row[kPassB];
#pragma unroll
    for (int p = 0; p < kPassB; ++p) {
        int r = row0 + ld_r + p * 32;
        r = r < a.n_rows ? r : a.n_rows - 1;
        const int64_t src = a.row_index ? a.row_index[r] : r;
        h_row[p] = a.hidden + src * a.row_stride;
    }
    const int n_kc = (a.d + BK - 1) / BK;
    const int n_groups = (a.m + BU - 1) / BU;
    const int total_it = n_groups * n_kc;

    uint4 stage[kPassA + kPassB];
    int ld_g = 0, ld_kc = 0;
    auto issue_loads = [&]() {
        const int k = ld_kc * BK + ld_c * 8;
        const bool k_ok = k < a.d;
#pragma unroll
        for (int p = 0; p < kPassA; ++p) {
            int u = ld_g * BU + ld_r + p * 32;
            u = u < a.m ? u : a.m - 1;
            stage[p] = k_ok ? *reinterpret_cast<const uint4*>(a.w1 + static_cast<int64_t>(u) * a.d + k) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int p = 0; p < kPassB; ++p)
            stage[kPassA + p] = k_ok ? *reinterpret_cast<const uint4*>(h_row[p] + k) : make_uint4(0, 0, 0, 0);
        if (++ld_kc == n_kc) { ld_kc = 0; ++ld_g; }
    };
    auto store_stage = [&](int buf) {
        unsigned char* sa = lds + buf * kStageBytes + ld_lds;
        unsigned char* sb = sa + BU * BK * 2;
#pragma unroll
        for (int p = 0; p < kPassA; ++p) *reinterpret_cast<uint4*>(sa + p * 32 * 128) = stage[p];
#pragma unroll
        for (int p = 0; p < kPassB; ++p) *reinterpret_cast<uint4*>(sb + p * 32 * 128) = stage[kPassA + p];
    };

    f32x16 acc[TU][TR];
#pragma unroll
    for (int c = 0; c < TU; ++c)
#pragma unroll
        for (int j = 0; j < TR; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[c][j][v] = 0.f;
    float part[TR] = {0.f, 0.f, 0.f, 0.f};   // this lane's share of s for rollout row0 + j*32 + l31

    const int swz = (l31 >> 1) & 7;
    issue_loads();
    store_stage(0);
    __syncthreads();
    int g = 0, kc = 0;
    for (int it = 0; it < total_it; ++it) {
        const bool more = it + 1 < total_it;
        if (more) issue_loads();
        const unsigned char* sa = lds + (it & 1) * kStageBytes;
        const unsigned char* sb = sa + BU * BK * 2;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int coff = ((kk * 2 + lh) ^ swz) << 4;
            bf16x8 fa[TU], fb[TR];
#pragma unroll
            for (int c = 0; c < TU; ++c)
                fa[c] = *reinterpret_cast<const bf16x8*>(sa + (c * 128 + wave * 32 + l31) * 128 + coff);
#pragma unroll
            for (int j = 0; j < TR; ++j)
                fb[j] = *reinterpret_cast<const bf16x8*>(sb + (j * 32 + l31) * 128 + coff);
#pragma unroll
            for (int c = 0; c < TU; ++c)
#pragma unroll
                for (int j = 0; j < TR; ++j)
                    acc[c][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c], fb[j], acc[c][j], 0, 0, 0);
        }
        if (more) store_stage((it + 1) & 1);
        __syncthreads();
        if (++kc == n_kc) {
            // acc[c][j][v] = pre-activation of unit g*BU + c*128 + wave*32 + (v/4)*8 + lh*4 + v%4
#pragma unroll
            for (int c = 0; c < TU; ++c)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int u = g * BU + c * 128 + wave * 32 + (v >> 2) * 8 + lh * 4 + (v & 3);
                    const bool live = u < a.m;
                    const float bias = (live && a.b1) ? a.b1[u] : 0.f;
                    const float w = live ? a.w2[u] : 0.f;
#pragma unroll
                    for (int j = 0; j < TR; ++j) {
                        part[j] = fmaf(fmaxf(acc[c][j][v] + bias, 0.f), w, part[j]);
                        acc[c][j][v] = 0.f;
                    }
                }
            kc = 0;
            ++g;
        }
    }
    // lane halves hold different units of the same rollout; then the four waves
#pragma unroll
    for (int j = 0; j < TR; ++j) part[j] += __shfl_xor(part[j], 32, ARROL_WAVE);
    float* red = reinterpret_cast<float*>(lds);   // [4 waves][BR]
    if (lh == 0) {
#pragma unroll
        for (int j = 0; j < TR; ++j) red[wave * BR + j * 32 + l31] = part[j];
    }
    __syncthreads();
    if (tid < BR && row0 + tid < a.n_rows) {
        const float s = red[tid] + red[BR + tid] + red[2 * BR + tid] + red[3 * BR + tid] + a.b2;
        float q;
        if (s >= 0.f) {
            q = 1.f / (1.f + expf(-s));
        } else {
            const float e = expf(s);
            q = e / (1.f + e);
        }
        if (a.score_out) a.score_out[row0 + tid] = s;
        a.prob_out[row0 + tid] = q;
    }
}

}  // namespace

extern "C" int arrol_score_mlp(const void* hidden, int64_t row_stride_elems, const int64_t* row_index,
                               const void* w1, const float* b1, const float* w2, float b2, int32_t n_rows,
                               int32_t d, int32_t m, float* score_out, float* prob_out, void* stream) {
    if (n_rows < 0 || d < 8 || (d & 7) || m < 1 || row_stride_elems < d || (row_stride_elems & 7)) return ARROL_EINVAL;
    if (n_rows == 0) return ARROL_OK;
    if (!hidden || !w1 || !w2 || !prob_out || !arrol_aligned16(hidden) || !arrol_aligned16(w1)) return ARROL_EINVAL;
    static bool lds_ok[64] = {};
    if (!arrol_allow_lds(&score_mlp_kernel, kLdsBytes, lds_ok)) return ARROL_EHIP;
    MlpArgs a;
    a.hidden = static_cast<const uint16_t*>(hidden); a.row_stride = row_stride_elems; a.row_index = row_index;
    a.w1 = static_cast<const uint16_t*>(w1); a.b1 = b1; a.w2 = w2; a.b2 = b2;
    a.n_rows = n_rows; a.d = d; a.m = m; a.score_out = score_out; a.prob_out = prob_out;
    hipLaunchKernelGGL(score_mlp_kernel, dim3((n_rows + BR - 1) / BR), dim3(kThreads), kLdsBytes,
                       static_cast<hipStream_t>(stream), a);
    return arrol_launch_status();
}
