// Training of the quality head (Sec. 4.2, Sec. 4.3 (iii), the optimizer step at the end of Alg. 1's frontend loop):
// cross-entropy loss of the linear head against the rollouts' rewards with its gradient, and an AdamW update.
// The hidden states are constants (the gradient stops at the backbone), so the gradient is one pass over the
// [N, d] matrix: HBM-streaming, every row read once and kept in registers between the forward dot product and
// the rank-one accumulation r_i * h_i.
#include "common.h"

namespace {

constexpr int kGradThreads = 512;
constexpr int kGradWaves = kGradThreads / ARROL_WAVE;
constexpr int kGradMaxBlocks = 1024;
constexpr int kGradMaxD = 8192;          // 16 chunks of 8 columns per lane

__device__ __forceinline__ void unpack8(const u32x4& x, float (&f)[8]) {
    f[0] = bf16_lo(x.x); f[1] = bf16_hi(x.x); f[2] = bf16_lo(x.y); f[3] = bf16_hi(x.y);
    f[4] = bf16_lo(x.z); f[5] = bf16_hi(x.z); f[6] = bf16_lo(x.w); f[7] = bf16_hi(x.w);
}

// One wavefront per row; lane l owns columns [8*(c*64+l), +8) for c < CH for every row it sees, so the
// gradient accumulators stay in its registers.  partial: [gridDim.x][d] fp32, tail: [gridDim.x][2] (loss, sum r).
template <int CH>
__global__ __launch_bounds__(kGradThreads) void score_grad_kernel(
    const u32x4* __restrict__ hidden, int64_t row_stride_vec, const int64_t* __restrict__ row_index,
    const float* __restrict__ w, float bias, const float* __restrict__ labels, int n_rows, int d_vec,
    float* __restrict__ partial, float* __restrict__ tail) {
    extern __shared__ float lds[];                 // d floats of head weights, then kGradWaves*512 floats
    float* w_lds = lds;
    float* red = lds + d_vec * 8;
    const int lane = threadIdx.x & (ARROL_WAVE - 1);
    const int wave = threadIdx.x / ARROL_WAVE;
    // the lane's slice of the weights lives in registers where that measured faster (2048 < d <= 4096: 4.2
    // against 3.9 TB/s; for smaller d the extra registers cost more occupancy than the LDS reads cost time:
    // 4.5 against 5.2 TB/s), otherwise the weights are read from LDS
    constexpr bool W_REG = CH == 8;
    constexpr int NW = W_REG ? CH : 1;
    float4 wra[NW], wrb[NW];
    if (W_REG) {
#pragma unroll
        for (int c = 0; c < NW; ++c) {
            const int v = c * ARROL_WAVE + lane;
            wra[c] = v < d_vec ? *reinterpret_cast<const float4*>(w + v * 8) : make_float4(0.f, 0.f, 0.f, 0.f);
            wrb[c] = v < d_vec ? *reinterpret_cast<const float4*>(w + v * 8 + 4) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    } else {
        for (int i = threadIdx.x; i < d_vec * 8; i += kGradThreads) w_lds[i] = w[i];
        __syncthreads();
    }
    float acc[CH][8];
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[c][k] = 0.f;
    float loss_acc = 0.f, r_acc = 0.f;
    const int wave_stride = gridDim.x * kGradWaves;
    for (int row = blockIdx.x * kGradWaves + wave; row < n_rows; row += wave_stride) {
        const int64_t src_row = row_index ? row_index[row] : row;
        const u32x4* p = hidden + src_row * row_stride_vec;
        u32x4 x[CH];
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int v = c * ARROL_WAVE + lane;
            x[c] = v < d_vec ? __builtin_nontemporal_load(p + v) : u32x4{0u, 0u, 0u, 0u};
        }
        float dot0 = 0.f, dot1 = 0.f;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int v = c * ARROL_WAVE + lane;
            if (v < d_vec) {
                const float4 wa = W_REG ? wra[W_REG ? c : 0] : *reinterpret_cast<const float4*>(w_lds + v * 8);
                const float4 wb = W_REG ? wrb[W_REG ? c : 0] : *reinterpret_cast<const float4*>(w_lds + v * 8 + 4);
                float f[8];
                unpack8(x[c], f);
                dot0 = fmaf(f[0], wa.x, dot0); dot1 = fmaf(f[1], wa.y, dot1);
                dot0 = fmaf(f[2], wa.z, dot0); dot1 = fmaf(f[3], wa.w, dot1);
                dot0 = fmaf(f[4], wb.x, dot0); dot1 = fmaf(f[5], wb.y, dot1);
                dot0 = fmaf(f[6], wb.z, dot0); dot1 = fmaf(f[7], wb.w, dot1);
            }
        }
        const float s = wave_sum_f32(dot0 + dot1) + bias;   // every lane holds the sum
        const float y = labels[row];
        const float e = expf(-fabsf(s));
        const float q = s >= 0.f ? 1.f / (1.f + e) : e / (1.f + e);
        const float r = q - y;
        // -[y log q + (1-y) log(1-q)] = max(s, 0) - y s + log(1 + exp(-|s|))
        loss_acc += fmaxf(s, 0.f) - y * s + log1pf(e);
        r_acc += r;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            float f[8];
            unpack8(x[c], f);
#pragma unroll
            for (int k = 0; k < 8; ++k) acc[c][k] = fmaf(r, f[k], acc[c][k]);
        }
    }
    // the workgroup's eight wavefronts add up through LDS, 512 columns at a time, in a fixed order
    float* out = partial + static_cast<int64_t>(blockIdx.x) * d_vec * 8;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        if (c * ARROL_WAVE < d_vec) {                          // uniform over the workgroup
            float* mine = red + wave * 512 + lane * 8;
            *reinterpret_cast<float4*>(mine) = make_float4(acc[c][0], acc[c][1], acc[c][2], acc[c][3]);
            *reinterpret_cast<float4*>(mine + 4) = make_float4(acc[c][4], acc[c][5], acc[c][6], acc[c][7]);
            __syncthreads();
            const int col = c * 512 + threadIdx.x;
            if (col < d_vec * 8) {
                float sum = 0.f;
#pragma unroll
                for (int k = 0; k < kGradWaves; ++k) sum += red[k * 512 + threadIdx.x];
                out[col] = sum;
            }
            __syncthreads();
        }
    }
    if (lane == 0) { red[wave * 2] = loss_acc; red[wave * 2 + 1] = r_acc; }
    __syncthreads();
    if (threadIdx.x < 2) {
        float sum = 0.f;
#pragma unroll
        for (int k = 0; k < kGradWaves; ++k) sum += red[k * 2 + threadIdx.x];
        tail[blockIdx.x * 2 + threadIdx.x] = sum;
    }
}

// Adds the per-workgroup partial sums in index order and divides by N.  Blocks 0 .. gridDim.x-2 cover the
// columns, the last block the loss and the bias gradient.
__global__ __launch_bounds__(256) void score_grad_reduce_kernel(
    const float* __restrict__ partial, const float* __restrict__ tail, int n_partials, int d, float inv_n,
    float* __restrict__ loss_out, float* __restrict__ grad_w, float* __restrict__ grad_bias) {
    if (blockIdx.x + 1 < gridDim.x) {
        const int col = blockIdx.x * 256 + threadIdx.x;
        if (col >= d) return;
        float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
        int p = 0;
        for (; p + 4 <= n_partials; p += 4) {
            s0 += partial[static_cast<int64_t>(p) * d + col];
            s1 += partial[static_cast<int64_t>(p + 1) * d + col];
            s2 += partial[static_cast<int64_t>(p + 2) * d + col];
            s3 += partial[static_cast<int64_t>(p + 3) * d + col];
        }
        for (; p < n_partials; ++p) s0 += partial[static_cast<int64_t>(p) * d + col];
        grad_w[col] = ((s0 + s1) + (s2 + s3)) * inv_n;
    } else if (threadIdx.x < ARROL_WAVE) {
        float a = 0.f, b = 0.f;
        for (int p = threadIdx.x; p < n_partials; p += ARROL_WAVE) { a += tail[p * 2]; b += tail[p * 2 + 1]; }
        a = wave_sum_f32(a);
        b = wave_sum_f32(b);
        if (threadIdx.x == 0) {
            if (loss_out) *loss_out = a * inv_n;
            if (grad_bias) *grad_bias = b * inv_n;
        }
    }
}

__global__ __launch_bounds__(256) void adamw_kernel(
    float* __restrict__ param, const float* __restrict__ grad, float* __restrict__ m, float* __restrict__ v,
    int64_t n, float lr, float beta1, float beta2, float eps, float weight_decay, float inv_bc1, float inv_bc2,
    uint16_t* __restrict__ param_bf16) {
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < n;
         i += static_cast<int64_t>(gridDim.x) * 256) {
        const float g = grad[i];
        const float mi = beta1 * m[i] + (1.f - beta1) * g;
        const float vi = beta2 * v[i] + (1.f - beta2) * g * g;
        m[i] = mi;
        v[i] = vi;
        const float p = param[i];
        const float upd = (mi * inv_bc1) / (sqrtf(vi * inv_bc2) + eps) + weight_decay * p;
        const float pn = p - lr * upd;
        param[i] = pn;
        if (param_bf16) param_bf16[i] = f32_to_bf16_rne(pn);
    }
}

int grad_blocks(int n_rows) {
    const int rows_per_block = kGradWaves * 8;
    int b = (n_rows + rows_per_block - 1) / rows_per_block;
    if (b > kGradMaxBlocks) b = kGradMaxBlocks;
    return b < 1 ? 1 : b;
}

template <int CH>
int launch_grad(int grid, size_t lds_bytes, hipStream_t st, const void* hidden, int64_t row_stride_vec,
                const int64_t* row_index, const float* w, float bias, const float* labels, int n_rows, int d_vec,
                float* partial, float* tail) {
    static arrol_device_flags lds_ok;
    if (!arrol_allow_lds(score_grad_kernel<CH>, static_cast<int>(sizeof(float) * (kGradMaxD + kGradWaves * 512)), lds_ok))
        return ARROL_EHIP;
    arrol_launch(score_grad_kernel<CH>, dim3(grid), dim3(kGradThreads), lds_bytes, st,
                       static_cast<const u32x4*>(hidden), row_stride_vec, row_index, w, bias, labels, n_rows, d_vec,
                       partial, tail);
    return arrol_launch_status();
}

}  // namespace

extern "C" size_t arrol_score_grad_workspace_bytes(int32_t n_rows, int32_t d) {
    if (n_rows < 0 || d < 8) return 0;
    return static_cast<size_t>(grad_blocks(n_rows)) * (static_cast<size_t>(d) + 2) * sizeof(float);
}

extern "C" int arrol_score_grad(const void* hidden, int64_t row_stride_elems, const int64_t* row_index,
                                const float* w, float bias, const float* labels, int32_t n_rows, int32_t d,
                                float* loss_out, float* grad_w, float* grad_bias, void* workspace,
                                size_t workspace_bytes, void* stream) {
    if (n_rows < 0 || d < 8 || (d & 7) || d > kGradMaxD || row_stride_elems < d || (row_stride_elems & 7))
        return ARROL_EINVAL;
    if (!grad_w) return ARROL_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int col_blocks = (d + 255) / 256;
    if (n_rows == 0) {   // empty batch: zero loss and gradients
        arrol_launch(score_grad_reduce_kernel, dim3(col_blocks + 1), dim3(256), 0, st, nullptr, nullptr, 0, d,
                           0.f, loss_out, grad_w, grad_bias);
        return arrol_launch_status();
    }
    if (!hidden || !w || !labels || !arrol_aligned16(hidden) || !arrol_aligned16(w)) return ARROL_EINVAL;
    if (!workspace || workspace_bytes < arrol_score_grad_workspace_bytes(n_rows, d)) return ARROL_EWORKSPACE;
    const int grid = grad_blocks(n_rows);
    float* partial = static_cast<float*>(workspace);
    float* tail = partial + static_cast<size_t>(grid) * d;
    const size_t lds_bytes = sizeof(float) * (static_cast<size_t>(d) + kGradWaves * 512);
    const int d_vec = d / 8;
    const int chunks = (d_vec + ARROL_WAVE - 1) / ARROL_WAVE;
    const int64_t rsv = row_stride_elems / 8;
    int rc;
    if (chunks <= 1) rc = launch_grad<1>(grid, lds_bytes, st, hidden, rsv, row_index, w, bias, labels, n_rows, d_vec, partial, tail);
    else if (chunks <= 2) rc = launch_grad<2>(grid, lds_bytes, st, hidden, rsv, row_index, w, bias, labels, n_rows, d_vec, partial, tail);
    else if (chunks <= 4) rc = launch_grad<4>(grid, lds_bytes, st, hidden, rsv, row_index, w, bias, labels, n_rows, d_vec, partial, tail);
    else if (chunks <= 8) rc = launch_grad<8>(grid, lds_bytes, st, hidden, rsv, row_index, w, bias, labels, n_rows, d_vec, partial, tail);
    else rc = launch_grad<16>(grid, lds_bytes, st, hidden, rsv, row_index, w, bias, labels, n_rows, d_vec, partial, tail);
    if (rc != ARROL_OK) return rc;
    arrol_launch(score_grad_reduce_kernel, dim3(col_blocks + 1), dim3(256), 0, st, partial, tail, grid, d,
                       1.f / static_cast<float>(n_rows), loss_out, grad_w, grad_bias);
    return arrol_launch_status();
}

extern "C" int arrol_adamw_step(float* param, const float* grad, float* m, float* v, int64_t n, int32_t step,
                                float lr, float beta1, float beta2, float eps, float weight_decay,
                                void* param_bf16, void* stream) {
    if (n < 0 || step < 1 || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f))
        return ARROL_EINVAL;
    if (n == 0) return ARROL_OK;
    if (!param || !grad || !m || !v) return ARROL_EINVAL;
    const double bc1 = 1.0 - __builtin_pow(static_cast<double>(beta1), static_cast<double>(step));
    const double bc2 = 1.0 - __builtin_pow(static_cast<double>(beta2), static_cast<double>(step));
    int64_t blocks = (n + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    arrol_launch(adamw_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), param, grad, m, v, n, lr, beta1, beta2, eps, weight_decay,
                       static_cast<float>(1.0 / bc1), static_cast<float>(1.0 / bc2),
                       static_cast<uint16_t*>(param_bf16));
    return arrol_launch_status();
}
