// GRPO on the surviving rollouts (Sec. 3 "Group-Relative Policy Optimization"; the frontend step of Alg. 1
// that follows the log-probs): the group-relative advantage and the clipped-ratio objective with its derivative
// with respect to the per-token log-probabilities that arrol_logprob produces.  A few bytes per token and a
// handful of groups: latency-bound kernels, written for fixed summation order and fp64 decisions rather than
// for bandwidth.
#include "common.h"

namespace {

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __longlong_as_double(shfl_xor_i64(__double_as_longlong(v), m));
    return v;
}

// one wavefront per group
__global__ __launch_bounds__(ARROL_WAVE) void grpo_advantage_kernel(
    const float* __restrict__ reward, const int64_t* __restrict__ group_offsets, int64_t N, int n_groups, int ddof,
    double eps, float* __restrict__ advantage, float* __restrict__ seq_weight) {
    const int g = blockIdx.x;
    int64_t lo = group_offsets[g], hi = group_offsets[g + 1];
    lo = lo < 0 ? 0 : (lo > N ? N : lo);
    hi = hi < lo ? lo : (hi > N ? N : hi);
    const int64_t n = hi - lo;
    if (n == 0) return;
    double s = 0.0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += ARROL_WAVE) s += static_cast<double>(reward[i]);
    const double mean = wave_sum_f64(s) / static_cast<double>(n);
    double q = 0.0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += ARROL_WAVE) {
        const double dv = static_cast<double>(reward[i]) - mean;
        q += dv * dv;
    }
    q = wave_sum_f64(q);
    const double stdv = n - ddof > 0 ? sqrt(q / static_cast<double>(n - ddof)) : 0.0;
    const double den = stdv + eps;
    const float wgt = static_cast<float>(1.0 / (static_cast<double>(n) * static_cast<double>(n_groups)));
    for (int64_t i = lo + threadIdx.x; i < hi; i += ARROL_WAVE) {
        const double dv = static_cast<double>(reward[i]) - mean;
        advantage[i] = den > 0.0 ? static_cast<float>(dv / den) : 0.f;
        if (seq_weight) seq_weight[i] = wgt;
    }
}

constexpr int kObjThreads = 256;
constexpr int kObjWaves = kObjThreads / ARROL_WAVE;

// one workgroup per rollout: partial[i] = weight_i * (1/L_i) * sum_t term_t, clipped[i] = tokens on the clipped branch
__global__ __launch_bounds__(kObjThreads) void grpo_objective_kernel(
    const float* __restrict__ logp, const float* __restrict__ logp_ref, const int64_t* __restrict__ cu, int64_t T,
    const float* __restrict__ advantage, const float* __restrict__ seq_weight, double eps_low, double eps_high,
    double beta, float* __restrict__ grad_logp, double* __restrict__ partial, int64_t* __restrict__ clipped) {
    __shared__ double sh_s[kObjWaves];
    __shared__ long long sh_c[kObjWaves];
    const int i = blockIdx.x;
    int64_t lo = cu[i], hi = cu[i + 1];
    lo = lo < 0 ? 0 : (lo > T ? T : lo);
    hi = hi < lo ? lo : (hi > T ? T : hi);
    const int64_t L = hi - lo;
    if (L == 0) {
        if (threadIdx.x == 0) { partial[i] = 0.0; clipped[i] = 0; }
        return;
    }
    const double A = static_cast<double>(advantage[i]);
    const double scale = static_cast<double>(seq_weight[i]) / static_cast<double>(L);
    const double r_lo = 1.0 - eps_low, r_hi = 1.0 + eps_high;
    double s = 0.0;
    long long c = 0;
    for (int64_t t = lo + threadIdx.x; t < hi; t += kObjThreads) {
        const double u = static_cast<double>(logp_ref[t]) - static_cast<double>(logp[t]);
        const double ratio = exp(-u);
        const double plain = ratio * A;
        const double clamped = fmin(fmax(ratio, r_lo), r_hi) * A;
        const double eu = exp(u);
        s += fmin(plain, clamped) - beta * (eu - u - 1.0);
        c += clamped < plain ? 1 : 0;
        if (grad_logp) {
            const double d = (plain <= clamped ? plain : 0.0) - beta * (1.0 - eu);
            grad_logp[t] = static_cast<float>(d * scale);
        }
    }
    s = wave_sum_f64(s);
    c = wave_sum_i64(c);
    const int lane = threadIdx.x & (ARROL_WAVE - 1), wave = threadIdx.x / ARROL_WAVE;
    if (lane == 0) { sh_s[wave] = s; sh_c[wave] = c; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double ts = 0.0;
        long long tc = 0;
        for (int w = 0; w < kObjWaves; ++w) { ts += sh_s[w]; tc += sh_c[w]; }
        partial[i] = ts * scale;
        clipped[i] = tc;
    }
}

// one workgroup: J = sum_i partial[i] in a fixed order
__global__ __launch_bounds__(kObjThreads) void grpo_finish_kernel(const double* __restrict__ partial,
                                                                  const int64_t* __restrict__ clipped, int n_seq,
                                                                  double* __restrict__ objective_out,
                                                                  int64_t* __restrict__ n_clipped) {
    __shared__ double sh_s[kObjWaves];
    __shared__ long long sh_c[kObjWaves];
    double s = 0.0;
    long long c = 0;
    for (int i = threadIdx.x; i < n_seq; i += kObjThreads) { s += partial[i]; c += clipped[i]; }
    s = wave_sum_f64(s);
    c = wave_sum_i64(c);
    const int lane = threadIdx.x & (ARROL_WAVE - 1), wave = threadIdx.x / ARROL_WAVE;
    if (lane == 0) { sh_s[wave] = s; sh_c[wave] = c; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double ts = 0.0;
        long long tc = 0;
        for (int w = 0; w < kObjWaves; ++w) { ts += sh_s[w]; tc += sh_c[w]; }
        if (objective_out) *objective_out = ts;
        if (n_clipped) *n_clipped = tc;
    }
}

}  // namespace

extern "C" int arrol_grpo_advantage(const float* reward, const int64_t* group_offsets, int64_t N, int32_t n_groups,
                                    int32_t ddof, float eps, float* advantage, float* seq_weight, void* stream) {
    if (N < 0 || n_groups < 0 || (ddof != 0 && ddof != 1) || !(eps >= 0.f)) return ARROL_EINVAL;
    if (n_groups == 0 || N == 0) return ARROL_OK;
    if (!reward || !group_offsets || !advantage) return ARROL_EINVAL;
    arrol_launch(grpo_advantage_kernel, dim3(n_groups), dim3(ARROL_WAVE), 0, static_cast<hipStream_t>(stream),
                       reward, group_offsets, N, n_groups, ddof, static_cast<double>(eps), advantage, seq_weight);
    return arrol_launch_status();
}

extern "C" size_t arrol_grpo_objective_workspace_bytes(int32_t n_seq) {
    return n_seq < 0 ? 0 : static_cast<size_t>(n_seq) * 16;
}

extern "C" int arrol_grpo_objective(const float* logp, const float* logp_ref, const int64_t* cu_seqlens, int64_t T,
                                    int32_t n_seq, const float* advantage, const float* seq_weight, float eps_low,
                                    float eps_high, float beta, double* objective_out, float* grad_logp,
                                    int64_t* n_clipped, void* workspace, size_t workspace_bytes, void* stream) {
    if (T < 0 || n_seq < 0 || !(eps_low >= 0.f && eps_low <= 1.f) || !(eps_high >= 0.f) || !(beta >= 0.f))
        return ARROL_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_seq == 0) {
        arrol_launch(grpo_finish_kernel, dim3(1), dim3(kObjThreads), 0, st, nullptr, nullptr, 0, objective_out,
                           n_clipped);
        return arrol_launch_status();
    }
    if (!cu_seqlens || !advantage || !seq_weight || (T > 0 && (!logp || !logp_ref))) return ARROL_EINVAL;
    if (!workspace || !arrol_aligned16(workspace) || workspace_bytes < arrol_grpo_objective_workspace_bytes(n_seq))
        return ARROL_EWORKSPACE;
    double* partial = static_cast<double*>(workspace);
    int64_t* clipped = reinterpret_cast<int64_t*>(partial + n_seq);
    arrol_launch(grpo_objective_kernel, dim3(n_seq), dim3(kObjThreads), 0, st, logp, logp_ref, cu_seqlens, T,
                       advantage, seq_weight, static_cast<double>(eps_low), static_cast<double>(eps_high),
                       static_cast<double>(beta), grad_logp, partial, clipped);
    arrol_launch(grpo_finish_kernel, dim3(1), dim3(kObjThreads), 0, st, partial, clipped, n_seq, objective_out,
                       n_clipped);
    return arrol_launch_status();
}
