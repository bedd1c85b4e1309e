// The paper's practical pruning policy (App. A.4 "Calibration Mapping and Survival Probability Design";
// Alg. 1, backend): binned posterior calibration of the sigmoid-normalised head score, survival
// probability with the keep-rate bias found by binary search, Bernoulli pruning with caller-supplied
// uniforms and an order-preserving stream compaction of the survivors.
#include "common.h"

namespace {

constexpr int kHistThreads = 256;
constexpr int kMaxBins = 2048;        // two fp64 tables of kMaxBins entries fit in LDS
constexpr int kCalThreads = 256;
constexpr int kPruneThreads = 1024;
constexpr int kBisectIters = 64;

// b(s') = min(B-1, floor(B s')), product in fp32 (App. A.4)
__device__ __forceinline__ int bin_of(float s_norm, int B) {
    int b = static_cast<int>(floorf(s_norm * static_cast<float>(B)));
    b = b < 0 ? 0 : b;
    return b < B - 1 ? b : B - 1;
}

__global__ void zero_counts_kernel(int64_t* c_pos, int64_t* c_neg, int B) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < B) { c_pos[i] = 0; c_neg[i] = 0; }
}

// Eq. 1: per-workgroup histograms in LDS, merged with 64-bit atomics (integer: order-free)
__global__ __launch_bounds__(kHistThreads) void histogram_kernel(
    const float* __restrict__ s_norm, const uint8_t* __restrict__ label, int64_t M, int B,
    unsigned long long* __restrict__ c_pos, unsigned long long* __restrict__ c_neg) {
    extern __shared__ unsigned int hist[];   // [2][B]
    for (int i = threadIdx.x; i < 2 * B; i += kHistThreads) hist[i] = 0;
    __syncthreads();
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kHistThreads;
    for (int64_t k = static_cast<int64_t>(blockIdx.x) * kHistThreads + threadIdx.x; k < M; k += stride)
        atomicAdd(&hist[(label[k] ? 0 : B) + bin_of(s_norm[k], B)], 1u);
    __syncthreads();
    for (int i = threadIdx.x; i < B; i += kHistThreads) {
        if (hist[i]) atomicAdd(&c_pos[i], static_cast<unsigned long long>(hist[i]));
        if (hist[B + i]) atomicAdd(&c_neg[i], static_cast<unsigned long long>(hist[B + i]));
    }
}

__device__ __forceinline__ double block_sum(double v, double* red) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        const long long o = shfl_xor_i64(__double_as_longlong(v), m);
        v += __longlong_as_double(o);
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) red[wave] = v;
    __syncthreads();
    double s = 0.0;
    for (int w = 0; w < kCalThreads / ARROL_WAVE; ++w) s += red[w];
    return s;
}

// Likelihoods, Bayes posterior, survival probability and the bisection for delta; one workgroup, fp64.
__global__ __launch_bounds__(kCalThreads) void calibrate_kernel(
    const int64_t* __restrict__ c_pos, const int64_t* __restrict__ c_neg, int B, arrol_policy pol,
    float* __restrict__ q_lut, float* __restrict__ p_lut, double* __restrict__ delta_out) {
    __shared__ double q_s[kMaxBins], w_s[kMaxBins];
    __shared__ double red[kCalThreads / ARROL_WAVE];
    const int tid = threadIdx.x;
    double np = 0.0, nn = 0.0;
    for (int b = tid; b < B; b += kCalThreads) { np += static_cast<double>(c_pos[b]); nn += static_cast<double>(c_neg[b]); }
    np = block_sum(np, red);
    nn = block_sum(nn, red);
    const double alpha = pol.alpha, kappa = pol.kappa, rho = pol.rho, lam = pol.lambda;
    const double p_min = pol.p_min, p_max = pol.p_max;
    const double pi = (np + nn) > 0.0 ? np / (np + nn) : 0.5;
    for (int b = tid; b < B; b += kCalThreads) {
        const double cp = static_cast<double>(c_pos[b]), cn = static_cast<double>(c_neg[b]);
        const double like_pos = (cp + alpha) / (np + alpha * B);
        const double like_neg = (cn + alpha) / (nn + alpha * B);
        const double num = pi * like_pos, den = num + (1.0 - pi) * like_neg;
        q_s[b] = den > 0.0 ? num / den : pi;
        w_s[b] = (np + nn) > 0.0 ? (cp + cn) / (np + nn) : 1.0 / B;
    }
    __syncthreads();
    double lo = p_min - kappa - lam, hi = p_max - kappa + lam;
    for (int it = 0; it < kBisectIters; ++it) {
        const double mid = 0.5 * (lo + hi);
        double e = 0.0;
        for (int b = tid; b < B; b += kCalThreads) {
            double p = kappa + mid + lam * (rho - q_s[b]);
            p = p < p_min ? p_min : (p > p_max ? p_max : p);
            e += w_s[b] * p;
        }
        e = block_sum(e, red);   // identical in every thread: the branch below is uniform
        if (e < kappa) lo = mid; else hi = mid;
    }
    const double delta = 0.5 * (lo + hi);
    for (int b = tid; b < B; b += kCalThreads) {
        double p = kappa + delta + lam * (rho - q_s[b]);
        p = p < p_min ? p_min : (p > p_max ? p_max : p);
        q_lut[b] = static_cast<float>(q_s[b]);
        p_lut[b] = static_cast<float>(p);
    }
    if (tid == 0 && delta_out) *delta_out = delta;
}

// Alg. 1: survival probability lookup, Bernoulli decision u < p, survivors compacted in rollout order
// (ballot + popcount inside a wave, LDS carry across waves and chunks).  One workgroup.
__global__ __launch_bounds__(kPruneThreads) void prune_bernoulli_kernel(
    const float* __restrict__ s_norm, const float* __restrict__ uniforms, int N, const float* __restrict__ p_lut,
    int B, float* __restrict__ p_out, uint8_t* __restrict__ keep_mask, int32_t* __restrict__ survivor_idx,
    int32_t* __restrict__ n_survivors) {
    __shared__ int wave_tot[kPruneThreads / ARROL_WAVE];
    __shared__ int carry_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry_s = 0;
    __syncthreads();
    for (int i0 = 0; i0 < N; i0 += kPruneThreads) {
        const int i = i0 + tid;
        bool keep = false;
        if (i < N) {
            const float p = p_lut[bin_of(s_norm[i], B)];
            keep = uniforms[i] < p;
            if (p_out) p_out[i] = p;
            keep_mask[i] = keep ? 1 : 0;
        }
        const uint64_t ballot = __ballot(keep);
        if (lane == 0) wave_tot[wave] = __popcll(ballot);
        __syncthreads();
        int before = carry_s;
        for (int w = 0; w < wave; ++w) before += wave_tot[w];
        if (keep) survivor_idx[before + __popcll(ballot & ((1ull << lane) - 1ull))] = i;
        __syncthreads();
        if (tid == kPruneThreads - 1) carry_s = before + __popcll(ballot);
        __syncthreads();
    }
    const int n = carry_s;
    for (int i = n + tid; i < N; i += kPruneThreads) survivor_idx[i] = -1;   // unused tail: "no rollout"
    if (tid == 0) *n_survivors = n;
}

bool policy_ok(const arrol_policy& p) {
    return p.kappa >= 0.f && p.kappa <= 1.f && p.rho >= 0.f && p.rho <= 1.f && p.lambda >= 0.f &&
           p.p_min >= 0.f && p.p_max <= 1.f && p.p_min <= p.p_max && p.alpha >= 0.f;
}

}  // namespace

extern "C" int arrol_histogram(const float* s_norm, const uint8_t* label, int64_t M, int32_t B,
                               int64_t* c_pos, int64_t* c_neg, void* stream) {
    if (M < 0 || B < 1 || B > kMaxBins || !c_pos || !c_neg) return ARROL_EINVAL;
    if (M > 0 && (!s_norm || !label)) return ARROL_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    arrol_launch(zero_counts_kernel, dim3((B + 255) / 256), dim3(256), 0, st, c_pos, c_neg, B);
    if (arrol_launch_failed()) return arrol_launch_status();
    if (M == 0) return ARROL_OK;
    int64_t blocks = (M + kHistThreads * 16 - 1) / (kHistThreads * 16);
    blocks = blocks < 1 ? 1 : (blocks > 1024 ? 1024 : blocks);
    arrol_launch(histogram_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kHistThreads),
                       2 * B * sizeof(unsigned int), st, s_norm, label, M, B,
                       reinterpret_cast<unsigned long long*>(c_pos), reinterpret_cast<unsigned long long*>(c_neg));
    return arrol_launch_status();
}

extern "C" int arrol_calibrate(const int64_t* c_pos, const int64_t* c_neg, int32_t B, arrol_policy pol,
                               float* q_lut, float* p_lut, double* delta, void* stream) {
    if (B < 1 || B > kMaxBins || !c_pos || !c_neg || !q_lut || !p_lut || !policy_ok(pol)) return ARROL_EINVAL;
    arrol_launch(calibrate_kernel, dim3(1), dim3(kCalThreads), 0, static_cast<hipStream_t>(stream), c_pos,
                       c_neg, B, pol, q_lut, p_lut, delta);
    return arrol_launch_status();
}

extern "C" int arrol_prune_bernoulli(const float* s_norm, const float* uniforms, int32_t N, const float* p_lut,
                                     int32_t B, float* p_out, uint8_t* keep_mask, int32_t* survivor_idx,
                                     int32_t* n_survivors, void* stream) {
    if (N < 0 || B < 1 || B > kMaxBins || !p_lut || !n_survivors) return ARROL_EINVAL;
    if (N > 0 && (!s_norm || !uniforms || !keep_mask || !survivor_idx)) return ARROL_EINVAL;
    arrol_launch(prune_bernoulli_kernel, dim3(1), dim3(kPruneThreads), 0, static_cast<hipStream_t>(stream),
                       s_norm, uniforms, N, p_lut, B, p_out, keep_mask, survivor_idx, n_survivors);
    return arrol_launch_status();
}
