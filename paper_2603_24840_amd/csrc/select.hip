// arrol_select: per-group keep-K selection by the balance rule of Thm 4.2 / App. A.1,
// applied G-K times to the shrinking group.  One wavefront per group, lane i owns rollout i.
// With S the live sum and n the live count, |mu_{-j} - rho| = |S - q_j - rho (n-1)| / (n-1),
// so each step prunes the live probability closest to t = S - rho (n-1); all of it in int64
// on the 2^-30 grid, hence order-free and identical on every machine.
#include "common.h"

namespace {

constexpr int kSelectThreads = 256;
constexpr int kGroupsPerBlock = kSelectThreads / ARROL_WAVE;

__global__ __launch_bounds__(kSelectThreads) void select_kernel(
    const float* __restrict__ prob, int n_groups, int G, int K, int64_t R,
    uint8_t* __restrict__ keep_mask, int32_t* __restrict__ survivor_idx) {
    const int lane = threadIdx.x & (ARROL_WAVE - 1);
    const int group = blockIdx.x * kGroupsPerBlock + threadIdx.x / ARROL_WAVE;
    if (group >= n_groups) return;  // whole wave leaves together
    bool live = lane < G;
    int64_t k = 0;
    if (live) k = static_cast<int64_t>(rintf(prob[static_cast<int64_t>(group) * G + lane] * 1073741824.0f));
    int64_t S = wave_sum_i64(k);
    for (int n = G; n > K; --n) {
        const int64_t t = S - R * (n - 1);
        int64_t dist = k - t;
        dist = dist < 0 ? -dist : dist;
        // (distance, lane) packed so that the minimum is the closest, lowest-index live lane
        const int64_t key = live ? ((dist << 6) | lane) : INT64_MAX;
        const int j = static_cast<int>(wave_min_i64(key) & 63);
        S -= shfl_i64(k, j);
        if (lane == j) live = false;
    }
    const uint64_t ballot = __ballot(live);
    if (lane < G) keep_mask[static_cast<int64_t>(group) * G + lane] = live ? 1 : 0;
    if (live) {
        const int rank = __popcll(ballot & ((1ull << lane) - 1ull));
        survivor_idx[static_cast<int64_t>(group) * K + rank] = group * G + lane;
    }
}

}  // namespace

extern "C" int arrol_select(const float* prob, int32_t n_groups, int32_t G, int32_t K, float rho,
                            uint8_t* keep_mask, int32_t* survivor_idx, void* stream) {
    if (n_groups < 0 || G < 1 || G > ARROL_MAX_GROUP || K < 1 || K > G) return ARROL_EINVAL;
    if (static_cast<int64_t>(n_groups) * G > INT32_MAX) return ARROL_EINVAL;
    if (!(rho >= 0.f && rho <= 1.f)) return ARROL_EINVAL;
    if (n_groups == 0) return ARROL_OK;
    if (!prob || !keep_mask || !survivor_idx) return ARROL_EINVAL;
    const int64_t R = static_cast<int64_t>(rintf(rho * 1073741824.0f));
    const int grid = (n_groups + kGroupsPerBlock - 1) / kGroupsPerBlock;
    arrol_launch(select_kernel, dim3(grid), dim3(kSelectThreads), 0, static_cast<hipStream_t>(stream),
                       prob, n_groups, G, K, R, keep_mask, survivor_idx);
    return arrol_launch_status();
}
