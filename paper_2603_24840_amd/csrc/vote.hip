// arrol_weighted_vote: rank-weighted answer vote (Sec. 4.4).  One wavefront per question,
// lane i owns candidate i.  Ranks are doubled average ranks, so everything after the fp32
// comparisons is integer and the result does not depend on candidate order.
#include "common.h"

namespace {

constexpr int kVoteThreads = 256;
constexpr int kQuestionsPerBlock = kVoteThreads / ARROL_WAVE;

__global__ __launch_bounds__(kVoteThreads) void vote_kernel(
    const float* __restrict__ prob, const int32_t* __restrict__ answer_id, int n_questions, int C,
    int n_answers, int32_t* __restrict__ winner, int64_t* __restrict__ tally) {
    const int lane = threadIdx.x & (ARROL_WAVE - 1);
    const int question = blockIdx.x * kQuestionsPerBlock + threadIdx.x / ARROL_WAVE;
    if (question >= n_questions) return;
    const int64_t base = static_cast<int64_t>(question) * C;
    const bool has = lane < C;
    const float q = has ? prob[base + lane] : 0.f;
    int ans = has ? answer_id[base + lane] : -1;
    if (ans < 0 || ans >= n_answers) ans = -1;  // takes no part
    int rank2 = 0;
    for (int j = 0; j < C; ++j) {
        const float qj = __shfl(q, j, ARROL_WAVE);
        rank2 += (qj < q ? 2 : 0) + ((qj == q && j != lane) ? 1 : 0);
    }
    // lanes sweep the answer ids 64 at a time; each keeps its best (tally, lowest id) key
    int64_t best = -1;
    for (int a0 = 0; a0 < n_answers; a0 += ARROL_WAVE) {
        const int a = a0 + lane;
        int64_t t = 0;
        bool occurs = false;
        for (int j = 0; j < C; ++j) {
            const int aj = __shfl(ans, j, ARROL_WAVE);
            const int rj = __shfl(rank2, j, ARROL_WAVE);
            if (aj == a) { t += rj; occurs = true; }
        }
        if (a < n_answers) {
            if (tally) tally[static_cast<int64_t>(question) * n_answers + a] = t;
            if (occurs) {
                const int64_t key = (t << 32) | static_cast<int64_t>(0x7fffffff - a);
                best = key > best ? key : best;
            }
        }
    }
    best = wave_max_i64(best);
    if (lane == 0) winner[question] = best < 0 ? -1 : static_cast<int32_t>(0x7fffffff - (best & 0x7fffffffll));
}

}  // namespace

extern "C" int arrol_weighted_vote(const float* prob, const int32_t* answer_id, int32_t n_questions,
                                   int32_t C, int32_t n_answers, int32_t* winner, int64_t* tally,
                                   void* stream) {
    if (n_questions < 0 || C < 1 || C > ARROL_MAX_GROUP || n_answers < 1) return ARROL_EINVAL;
    if (n_questions == 0) return ARROL_OK;
    if (!prob || !answer_id || !winner) return ARROL_EINVAL;
    const int grid = (n_questions + kQuestionsPerBlock - 1) / kQuestionsPerBlock;
    arrol_launch(vote_kernel, dim3(grid), dim3(kVoteThreads), 0, static_cast<hipStream_t>(stream),
                       prob, answer_id, n_questions, C, n_answers, winner, tally);
    return arrol_launch_status();
}
