// Trace confidence (Sec. 3 "Trace Confidence"): token confidence H_t = -sum_j log P_t(j) and its trace-level
// aggregates (trace mean, sliding-window means, their minimum and the mean of the lowest share of windows).
//
// With z_t = W h_t and lse_t = logsumexp_j z_t[j] (an output of the fused log-prob kernel):
//     H_t = V * lse_t - sum_j z_t[j] = V * lse_t - <h_t, sum_j W_j>
// so beside the log-prob pass the token confidence costs one column sum of the LM head (HBM stream over W,
// once per weight version) and one dot product per token (HBM stream over the hidden states): no second
// [T, V] contraction.  The aggregates run one workgroup per trace in fp64.
#include "common.h"

namespace {

constexpr int kColThreads = 256;
constexpr int kColRows = 256;      // LM-head rows per workgroup of the column-sum pass
constexpr int kColUnroll = 8;

// partial[b][c] = sum of W[v][c] over the rows v of block b
__global__ __launch_bounds__(kColThreads) void colsum_partial_kernel(
    const u32x4* __restrict__ lm_head, int V, int d_vec, float* __restrict__ partial) {
    const int v0 = blockIdx.x * kColRows;
    const int v1 = v0 + kColRows < V ? v0 + kColRows : V;
    for (int c = threadIdx.x; c < d_vec; c += kColThreads) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        const u32x4* p = lm_head + c;
        for (int v = v0; v < v1; v += kColUnroll) {
            u32x4 x[kColUnroll];
#pragma unroll
            for (int u = 0; u < kColUnroll; ++u)
                x[u] = v + u < v1 ? __builtin_nontemporal_load(p + static_cast<int64_t>(v + u) * d_vec)
                                  : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
            for (int u = 0; u < kColUnroll; ++u) {
                acc[0] += bf16_lo(x[u].x); acc[1] += bf16_hi(x[u].x);
                acc[2] += bf16_lo(x[u].y); acc[3] += bf16_hi(x[u].y);
                acc[4] += bf16_lo(x[u].z); acc[5] += bf16_hi(x[u].z);
                acc[6] += bf16_lo(x[u].w); acc[7] += bf16_hi(x[u].w);
            }
        }
        float* out = partial + (static_cast<int64_t>(blockIdx.x) * d_vec + c) * 8;
        *reinterpret_cast<float4*>(out) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        *reinterpret_cast<float4*>(out + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
    }
}

constexpr int kConfThreads = 512;
constexpr int kConfWaves = kConfThreads / ARROL_WAVE;
constexpr int kConfUnroll = 4;

// one wavefront per token: conf[t] = V * lse[t] - <h_t, colsum>.  CH > 0: lane l owns chunks c*64 + l (c < CH) of
// every row and keeps its slice of colsum in registers (d <= 512*CH); CH == 0: colsum staged in LDS, any d.
template <int CH>
__global__ __launch_bounds__(kConfThreads) void token_conf_kernel(
    const u32x4* __restrict__ hidden, const float* __restrict__ colsum, const float* __restrict__ lse,
    int64_t T, int V, int d_vec, float* __restrict__ conf) {
    extern __shared__ float c_lds[];
    const int lane = threadIdx.x & (ARROL_WAVE - 1);
    const int wave = threadIdx.x / ARROL_WAVE;
    constexpr int NR = CH > 0 ? CH : 1;
    float4 wa[NR], wb[NR];
    if (CH > 0) {
#pragma unroll
        for (int c = 0; c < NR; ++c) {
            const int v = c * ARROL_WAVE + lane;
            wa[c] = v < d_vec ? *reinterpret_cast<const float4*>(colsum + v * 8) : make_float4(0.f, 0.f, 0.f, 0.f);
            wb[c] = v < d_vec ? *reinterpret_cast<const float4*>(colsum + v * 8 + 4) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    } else {
        for (int i = threadIdx.x; i < d_vec * 8; i += kConfThreads) c_lds[i] = colsum[i];
        __syncthreads();
    }
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kConfWaves;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kConfWaves + wave; t < T; t += stride) {
        const u32x4* p = hidden + t * d_vec;
        float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
        if (CH > 0) {
            u32x4 x[NR];
#pragma unroll
            for (int c = 0; c < NR; ++c) {
                const int v = c * ARROL_WAVE + lane;
                x[c] = v < d_vec ? __builtin_nontemporal_load(p + v) : u32x4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int c = 0; c < NR; ++c) {
                acc0 = fmaf(bf16_lo(x[c].x), wa[c].x, acc0); acc1 = fmaf(bf16_hi(x[c].x), wa[c].y, acc1);
                acc2 = fmaf(bf16_lo(x[c].y), wa[c].z, acc2); acc3 = fmaf(bf16_hi(x[c].y), wa[c].w, acc3);
                acc0 = fmaf(bf16_lo(x[c].z), wb[c].x, acc0); acc1 = fmaf(bf16_hi(x[c].z), wb[c].y, acc1);
                acc2 = fmaf(bf16_lo(x[c].w), wb[c].z, acc2); acc3 = fmaf(bf16_hi(x[c].w), wb[c].w, acc3);
            }
        } else {
            for (int v0 = 0; v0 < d_vec; v0 += kConfUnroll * ARROL_WAVE) {
                u32x4 x[kConfUnroll];
#pragma unroll
                for (int u = 0; u < kConfUnroll; ++u) {
                    const int v = v0 + u * ARROL_WAVE + lane;
                    x[u] = v < d_vec ? __builtin_nontemporal_load(p + v) : u32x4{0u, 0u, 0u, 0u};
                }
#pragma unroll
                for (int u = 0; u < kConfUnroll; ++u) {
                    const int v = v0 + u * ARROL_WAVE + lane;
                    if (v < d_vec) {
                        const float4 la = *reinterpret_cast<const float4*>(c_lds + v * 8);
                        const float4 lb = *reinterpret_cast<const float4*>(c_lds + v * 8 + 4);
                        acc0 = fmaf(bf16_lo(x[u].x), la.x, acc0); acc1 = fmaf(bf16_hi(x[u].x), la.y, acc1);
                        acc2 = fmaf(bf16_lo(x[u].y), la.z, acc2); acc3 = fmaf(bf16_hi(x[u].y), la.w, acc3);
                        acc0 = fmaf(bf16_lo(x[u].z), lb.x, acc0); acc1 = fmaf(bf16_hi(x[u].z), lb.y, acc1);
                        acc2 = fmaf(bf16_lo(x[u].w), lb.z, acc2); acc3 = fmaf(bf16_hi(x[u].w), lb.w, acc3);
                    }
                }
            }
        }
        const float dot = wave_sum_f32((acc0 + acc1) + (acc2 + acc3));
        if (lane == 0)
            conf[t] = static_cast<float>(static_cast<double>(V) * static_cast<double>(lse[t]) -
                                         static_cast<double>(dot));
    }
}

// ---- trace-level aggregates -------------------------------------------------------------------------------
constexpr int kAggThreads = 256;
constexpr int kAggWaves = kAggThreads / ARROL_WAVE;
constexpr int kAggItems = 8;       // tokens per thread per scan chunk

__device__ __forceinline__ double shfl_up_f64(double v, int delta) {
    const int64_t b = __double_as_longlong(v);
    const int lo = __shfl_up(static_cast<int>(b & 0xffffffffll), delta, ARROL_WAVE);
    const int hi = __shfl_up(static_cast<int>(b >> 32), delta, ARROL_WAVE);
    return __longlong_as_double((static_cast<int64_t>(hi) << 32) | static_cast<uint32_t>(lo));
}
__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __longlong_as_double(shfl_xor_i64(__double_as_longlong(v), m));
    return v;
}
// order-preserving map of a double onto unsigned integers
__device__ __forceinline__ uint64_t key_of(double v) {
    const uint64_t b = static_cast<uint64_t>(__double_as_longlong(v));
    return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}
__device__ __forceinline__ double value_of(uint64_t k) {
    const uint64_t b = (k >> 63) ? (k & 0x7fffffffffffffffull) : ~k;
    return __longlong_as_double(static_cast<int64_t>(b));
}

// One workgroup per trace.  prefix and keys are per-trace slices of the workspace: trace i owns entries
// [cu[i] + i, cu[i+1] + i + 1) of each (L+1 prefix sums, up to L window keys).
__global__ __launch_bounds__(kAggThreads) void trace_conf_kernel(
    const float* __restrict__ conf, const int64_t* __restrict__ cu, int64_t T, int window, int bottom_percent,
    double* __restrict__ prefix_all, uint64_t* __restrict__ keys_all, double* __restrict__ mean_out,
    double* __restrict__ min_out, double* __restrict__ bottom_out) {
    __shared__ double sh_d[2][kAggWaves];
    __shared__ unsigned long long sh_u[2][kAggWaves];
    const int i = blockIdx.x;
    const int lane = threadIdx.x & (ARROL_WAVE - 1), wave = threadIdx.x / ARROL_WAVE;
    int64_t lo = cu[i], hi = cu[i + 1];
    lo = lo < 0 ? 0 : (lo > T ? T : lo);
    hi = hi < lo ? lo : (hi > T ? T : hi);
    const int64_t L = hi - lo;
    const double nan = __longlong_as_double(0x7ff8000000000000ll);
    if (L == 0) {
        if (threadIdx.x == 0) { mean_out[i] = nan; min_out[i] = nan; bottom_out[i] = nan; }
        return;
    }
    double* prefix = prefix_all + lo + i;
    uint64_t* keys = keys_all + lo + i;
    const float* x = conf + lo;

    // ---- inclusive prefix sums in fp64, 2048 tokens per round
    double carry = 0.0;
    if (threadIdx.x == 0) prefix[0] = 0.0;
    int par = 0;
    for (int64_t base = 0; base < L; base += kAggThreads * kAggItems, par ^= 1) {
        const int64_t first = base + static_cast<int64_t>(threadIdx.x) * kAggItems;
        double v[kAggItems];
        double run = 0.0;
#pragma unroll
        for (int k = 0; k < kAggItems; ++k) {
            run += first + k < L ? static_cast<double>(x[first + k]) : 0.0;
            v[k] = run;
        }
        double incl = run;                              // inclusive scan of the thread totals over the wave
#pragma unroll
        for (int dlt = 1; dlt < ARROL_WAVE; dlt <<= 1) {
            const double o = shfl_up_f64(incl, dlt);
            if (lane >= dlt) incl += o;
        }
        if (lane == ARROL_WAVE - 1) sh_d[par][wave] = incl;
        __syncthreads();
        double before = carry, total = carry;
#pragma unroll
        for (int w = 0; w < kAggWaves; ++w) {
            const double s = sh_d[par][w];
            if (w < wave) before += s;
            total += s;
        }
        const double offset = before + (incl - run);
#pragma unroll
        for (int k = 0; k < kAggItems; ++k)
            if (first + k < L) prefix[first + k + 1] = offset + v[k];
        carry = total;
    }
    __syncthreads();                                    // prefix[] of this trace is complete and visible

    // ---- window means, their keys, the minimum
    const int64_t w_eff = window < L ? window : L;
    const int64_t n_w = L - w_eff + 1;
    const double inv_w = 1.0 / static_cast<double>(w_eff);
    uint64_t kmin = ~0ull;
    for (int64_t k = threadIdx.x; k < n_w; k += kAggThreads) {
        const uint64_t key = key_of((prefix[k + w_eff] - prefix[k]) * inv_w);
        keys[k] = key;
        kmin = key < kmin ? key : kmin;
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        const uint64_t o = static_cast<uint64_t>(shfl_xor_i64(static_cast<int64_t>(kmin), m));
        kmin = o < kmin ? o : kmin;
    }
    if (lane == 0) sh_u[0][wave] = kmin;
    __syncthreads();                                    // also orders keys[] before the passes below
    kmin = sh_u[0][0];
#pragma unroll
    for (int w = 1; w < kAggWaves; ++w) kmin = sh_u[0][w] < kmin ? sh_u[0][w] : kmin;

    // ---- the m-th smallest window key, bit by bit: the largest X with #{key < X} < m
    const int64_t m_low = (n_w * bottom_percent + 99) / 100 < 1 ? 1 : (n_w * bottom_percent + 99) / 100;
    uint64_t X = 0;
    par = 1;
    for (int b = 63; b >= 0; --b, par ^= 1) {
        const uint64_t cand = X | (1ull << b);
        unsigned long long cnt = 0;
        for (int64_t k = threadIdx.x; k < n_w; k += kAggThreads) cnt += keys[k] < cand ? 1u : 0u;
        cnt = static_cast<unsigned long long>(wave_sum_i64(static_cast<int64_t>(cnt)));
        if (lane == 0) sh_u[par][wave] = cnt;
        __syncthreads();
        unsigned long long tot = 0;
#pragma unroll
        for (int w = 0; w < kAggWaves; ++w) tot += sh_u[par][w];
        if (static_cast<int64_t>(tot) < m_low) X = cand;
    }
    // sum of the values below X, then as many copies of X as are still missing
    double s_low = 0.0;
    unsigned long long c_low = 0;
    for (int64_t k = threadIdx.x; k < n_w; k += kAggThreads) {
        const uint64_t key = keys[k];
        if (key < X) { s_low += value_of(key); ++c_low; }
    }
    s_low = wave_sum_f64(s_low);
    c_low = static_cast<unsigned long long>(wave_sum_i64(static_cast<int64_t>(c_low)));
    __syncthreads();
    if (lane == 0) { sh_d[0][wave] = s_low; sh_u[0][wave] = c_low; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
        unsigned long long c = 0;
        for (int w = 0; w < kAggWaves; ++w) { s += sh_d[0][w]; c += sh_u[0][w]; }
        s += static_cast<double>(m_low - static_cast<int64_t>(c)) * value_of(X);
        mean_out[i] = prefix[L] / static_cast<double>(L);
        min_out[i] = value_of(kmin);
        bottom_out[i] = s / static_cast<double>(m_low);
    }
}

int colsum_blocks(int V) { return (V + kColRows - 1) / kColRows; }

}  // namespace

extern "C" size_t arrol_token_confidence_workspace_bytes(int32_t V, int32_t d) {
    if (V < 1 || d < 8) return 0;
    return (static_cast<size_t>(colsum_blocks(V)) + 1) * static_cast<size_t>(d) * sizeof(float);
}

extern "C" int arrol_token_confidence(const void* hidden, const void* lm_head, const float* lse, int64_t T,
                                      int32_t V, int32_t d, float* conf_out, void* workspace,
                                      size_t workspace_bytes, void* stream) {
    if (T < 0 || V < 1 || d < 8 || (d & 7) || d > 16384) return ARROL_EINVAL;
    if (T == 0) return ARROL_OK;
    if (!hidden || !lm_head || !lse || !conf_out || !arrol_aligned16(hidden) || !arrol_aligned16(lm_head))
        return ARROL_EINVAL;
    if (!workspace || !arrol_aligned16(workspace) || workspace_bytes < arrol_token_confidence_workspace_bytes(V, d))
        return ARROL_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int nb = colsum_blocks(V);
    float* colsum = static_cast<float*>(workspace);
    float* partial = colsum + d;
    arrol_launch(colsum_partial_kernel, dim3(nb), dim3(kColThreads), 0, st,
                       static_cast<const u32x4*>(lm_head), V, d / 8, partial);
    arrol_launch(reduce_rows_f32_kernel<0>, dim3((d + 31) / 32), dim3(256), 0, st, partial, nb,
                       static_cast<int64_t>(d), static_cast<int64_t>(d), 1.f, colsum);
    const int64_t blocks_needed = (T + kConfWaves - 1) / kConfWaves;
    const int grid = static_cast<int>(blocks_needed < 256 * 8 ? blocks_needed : 256 * 8);
    const u32x4* h = static_cast<const u32x4*>(hidden);
    const int chunks = (d / 8 + ARROL_WAVE - 1) / ARROL_WAVE;
#define ARROL_CONF(CH, LDS) arrol_launch(token_conf_kernel<CH>, dim3(grid), dim3(kConfThreads), LDS, st, h, colsum, lse, T, V, d / 8, conf_out)
    if (chunks <= 1) ARROL_CONF(1, 0);
    else if (chunks <= 2) ARROL_CONF(2, 0);
    else if (chunks <= 4) ARROL_CONF(4, 0);
    else if (chunks <= 8) ARROL_CONF(8, 0);
    else {
        static arrol_device_flags lds_ok;
        if (!arrol_allow_lds(token_conf_kernel<0>, static_cast<int>(sizeof(float) * 16384), lds_ok)) return ARROL_EHIP;
        ARROL_CONF(0, sizeof(float) * d);
    }
#undef ARROL_CONF
    return arrol_launch_status();
}

extern "C" size_t arrol_trace_confidence_workspace_bytes(int64_t T, int32_t n_seq) {
    if (T < 0 || n_seq < 0) return 0;
    return 2 * (static_cast<size_t>(T) + static_cast<size_t>(n_seq)) * sizeof(double);
}

extern "C" int arrol_trace_confidence(const float* conf, const int64_t* cu_seqlens, int64_t T, int32_t n_seq,
                                      int32_t window, int32_t bottom_percent, double* mean_out,
                                      double* min_out, double* bottom_out, void* workspace,
                                      size_t workspace_bytes, void* stream) {
    if (T < 0 || n_seq < 0 || window < 1 || bottom_percent < 1 || bottom_percent > 100) return ARROL_EINVAL;
    if (n_seq == 0) return ARROL_OK;
    if (!cu_seqlens || !mean_out || !min_out || !bottom_out || (T > 0 && !conf)) return ARROL_EINVAL;
    if (!workspace || !arrol_aligned16(workspace) || workspace_bytes < arrol_trace_confidence_workspace_bytes(T, n_seq))
        return ARROL_EWORKSPACE;
    double* prefix = static_cast<double*>(workspace);
    uint64_t* keys = reinterpret_cast<uint64_t*>(prefix + T + n_seq);
    arrol_launch(trace_conf_kernel, dim3(n_seq), dim3(kAggThreads), 0, static_cast<hipStream_t>(stream), conf,
                       cu_seqlens, T, window, bottom_percent, prefix, keys, mean_out, min_out, bottom_out);
    return arrol_launch_status();
}
