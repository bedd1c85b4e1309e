/*
 * arrol.h -- C ABI of the ARRoL online rollout-pruning data path for AMD MI355X (gfx950).
 *
 * Method: "Prune as You Generate: Online Rollout Pruning for Faster and Better RLVR".
 * The five calls are the stages of the in-engine pruning path:
 *   arrol_score          quality head on checkpoint hidden states + sigmoid   (Sec. 4.2, App. A.4)
 *   arrol_select         exactly-K correctness-balanced survivors per group   (Sec. 4.1, Thm 4.2, App. A.1)
 *   arrol_compact        gather survivors' paged KV cache / tokens, re-batch  (Sec. 4.3 (i),(ii); Alg. 1)
 *   arrol_logprob        per-token log pi(o_t | o_<t) on the survivors        (Sec. 3 GRPO ratio; Sec. 4.3 (ii); Alg. 1)
 *   arrol_weighted_vote  rank-weighted answer vote for test-time scaling      (Sec. 4.4)
 * plus, around them:
 *   arrol_histogram, arrol_calibrate, arrol_prune_bernoulli   the paper's practical stochastic policy (App. A.4 Eq. 1-2; Alg. 1)
 *   arrol_score_mlp                                            the 2-layer MLP form of the quality head (Sec. 4.2)
 *   arrol_score_grad, arrol_score_mlp_grad, arrol_adamw_step  training the head on the fly (Sec. 4.2, 4.3 (iii); Alg. 1)
 *   arrol_compact_inplace                                      hole-filling compaction of the same pool (Sec. 4.3 (i))
 *   arrol_compact_static                                       arrol_compact without a workspace argument (fixed scratch)
 *   arrol_probe_mfma_rate                                      measurement aid: register-only bf16 MFMA rate of this card
 *   arrol_token_confidence, arrol_trace_confidence             trace confidence (Sec. 3)
 *   arrol_grpo_advantage, arrol_grpo_objective                 group-relative advantage, clipped objective (Sec. 3)
 *
 * Conventions common to every call
 *   - Every data pointer is a DEVICE pointer owned by the caller (the library never
 *     allocates, frees or keeps one).  Scratch memory is passed in as `workspace`;
 *     its size comes from the matching *_workspace_bytes() query (a host computation).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue kernels on it: no host synchronisation, no device-to-host copy.
 *   - Return value: ARROL_OK, or a negative ARROL_E* code.  Argument and workspace errors
 *     (ARROL_EINVAL, ARROL_EWORKSPACE) are detected on the host before anything is launched:
 *     nothing has been enqueued.  ARROL_EHIP means the runtime refused a launch; a call made
 *     of several launches may then have enqueued the earlier ones, and its outputs are undefined.
 *   - Every kernel stays inside the buffers described here for ANY contents of the index
 *     arrays whose range the call is told (block tables, survivor ids, targets, offsets:
 *     out-of-range entries are skipped or clamped, see each call).  The one exception is
 *     row_index of the scoring calls: the library is not told how many rows `hidden` holds,
 *     so every row_index[i] must address a row of the caller's buffer.
 */
#ifndef ARROL_H
#define ARROL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ARROL_OK 0
#define ARROL_EINVAL (-1)     /* null pointer, bad shape, misaligned base */
#define ARROL_EWORKSPACE (-2) /* workspace missing or too small */
#define ARROL_EHIP (-3)       /* the HIP runtime refused a launch */

#define ARROL_MAX_GROUP 64      /* largest G (arrol_select) and C (arrol_weighted_vote) */
#define ARROL_FIXED_POINT_BITS 30

/* Library version (major*10000 + minor*100 + patch); changes whenever an argument list of this header does. */
int arrol_version(void);
/* Static, NUL-terminated description of a return code. */
const char* arrol_error_string(int code);

/*
 * Stage 1 -- quality head and success probability (Sec. 4.2 "Quality Score Prediction";
 * App. A.4: the score is squashed to [0,1] with the sigmoid).
 *   s_i = <w, h_i> + bias,  q_i = 1 / (1 + exp(-s_i))
 * hidden     bf16 [*, d], row r starts at hidden + r*row_stride_elems (elements);
 *            row_stride_elems >= d and a multiple of 8; base 16-byte aligned.
 * row_index  NULL, or int64 [n_rows]: output i reads row row_index[i] (lets the caller
 *            point into a token-major buffer); NULL means row i.
 * w          fp32 [d]; bias fp32 by value.  d must be a multiple of 8, d >= 8.
 * score_out  NULL or fp32 [n_rows] (s_i); prob_out fp32 [n_rows] (q_i).
 * fp32 accumulation of exact bf16 x fp32 products.  n_rows == 0 is a no-op.
 */
int arrol_score(const void* hidden, int64_t row_stride_elems, const int64_t* row_index,
                const float* w, float bias, int32_t n_rows, int32_t d,
                float* score_out, float* prob_out, void* stream);

/*
 * Stage 1, MLP head (Sec. 4.2 allows a small two-layer MLP as the quality head; neither width nor
 * activation is given - ReLU is this build's reading):
 *   a = relu(W1 h + b1),  s_i = <w2, a> + b2,  q_i = sigmoid(s_i)
 * hidden, row_stride_elems, row_index, score_out, prob_out as in arrol_score.
 * w1 bf16 [m, d] row-major, 16-byte aligned; b1 NULL (zero) or fp32 [m]; w2 fp32 [m]; b2 by value; m >= 1.
 * bf16 products accumulated in fp32 on the matrix cores; the [n_rows, m] activations are never stored.
 * workspace: optional.  With NULL (or fewer than arrol_score_mlp_workspace_bytes(n_rows, d, m) bytes) the
 * call is one kernel whose workgroups each take 128 rollouts; given the queried size (16-byte aligned) a
 * small batch (the query returns 0 where this does not apply) is spread over the whole GPU instead - one
 * wavefront per 32 units x 32 rollouts, partial sums over the units in the workspace, added in a fixed
 * order by a second launch.  Results of the two paths differ by fp32 summation order only.
 */
size_t arrol_score_mlp_workspace_bytes(int32_t n_rows, int32_t d, int32_t m);
int arrol_score_mlp(const void* hidden, int64_t row_stride_elems, const int64_t* row_index,
                    const void* w1, const float* b1, const float* w2, float b2, int32_t n_rows,
                    int32_t d, int32_t m, float* score_out, float* prob_out, void* workspace,
                    size_t workspace_bytes, void* stream);

/*
 * Stage 2 -- per-group keep-K selection by the balance rule (Thm 4.2 / App. A.1):
 * with live set A, mu_{-j} = mean of q_i over A \ {j}; prune argmin_j |mu_{-j} - rho|;
 * repeat on the shrunken group until K remain.  Decisions are taken on integers
 * k_i = rint(q_i * 2^30) (round-half-even of the fp32 value) and R = rint(rho * 2^30),
 * so the result is the same on any hardware; ties prune the lowest index.
 * prob          fp32 [n_groups*G], finite, in [0,1]; groups are consecutive runs of G.
 * keep_mask     uint8 [n_groups*G]  1 = survivor.
 * survivor_idx  int32 [n_groups*K]  global rollout ids, ascending.
 * Requires 1 <= K <= G <= ARROL_MAX_GROUP.  n_groups == 0 is a no-op.
 */
int arrol_select(const float* prob, int32_t n_groups, int32_t G, int32_t K, float rho,
                 uint8_t* keep_mask, int32_t* survivor_idx, void* stream);

/*
 * Paged KV pool geometry.  Memory order is [layer][K|V][page][token][kv_head][dim], bf16,
 * i.e. one (layer, K|V, page) chunk is page_tokens*n_kv_heads*head_dim*2 contiguous bytes.
 */
typedef struct arrol_kv_layout {
    int32_t n_layers;
    int32_t page_tokens;
    int32_t n_kv_heads;
    int32_t head_dim;
    int64_t n_pages; /* pages per (layer, K|V) slab in THIS pool */
} arrol_kv_layout;

/*
 * Stage 3 -- compaction / re-batch (Sec. 4.3 (i): pruned requests leave the pool so their
 * capacity is reused; (ii) and the frontend step of Alg. 1 that drops the pruned rollouts and re-batches the rest).
 * Survivor rank r (r-th entry of survivor_idx, source rollout s) owns
 * np_r = min(ceil(seq_len_src[s] / page_tokens), max_pages_per_seq) destination pages
 * starting at base_r = sum_{r' < r} np_r'.  For every layer and K|V the source page
 * block_table_src[s][p] is copied verbatim (whole page) to destination page base_r + p.
 *   block_table_dst[r][p] = base_r + p (p < np_r), -1 otherwise;  seq_len_dst[r] = seq_len_src[s];
 *   tokens_dst[r][:] = tokens_src[s][:];  src_of_dst[r] = s;  *n_pages_used = base_{n_keep}.
 * Source and destination pools must agree in everything but n_pages and must not overlap.
 * The chunk size (bytes) must be a multiple of 16 and both pool bases 16-byte aligned.
 * A survivor id outside [0, n_src) gives an empty destination rollout (np_r = 0, seq_len 0,
 * src_of_dst -1, tokens row of zeros); a source page id outside [0, src.n_pages) or a
 * destination page >= dst.n_pages is skipped (the caller can detect overflow from
 * *n_pages_used > dst.n_pages).  Destination pages >= *n_pages_used are left untouched.
 * tokens_src/tokens_dst may both be NULL (max_len ignored).  n_keep == 0 only writes
 * *n_pages_used = 0.
 * workspace: arrol_compact_workspace_bytes(n_keep) bytes, 16-byte aligned.
 */
size_t arrol_compact_workspace_bytes(int32_t n_keep);
int arrol_compact(const void* kv_src, arrol_kv_layout src, void* kv_dst, arrol_kv_layout dst,
                  const int32_t* block_table_src, const int32_t* seq_len_src,
                  int32_t max_pages_per_seq, const int32_t* tokens_src, int32_t max_len,
                  const int32_t* survivor_idx, int32_t n_src, int32_t n_keep,
                  int32_t* block_table_dst, int32_t* seq_len_dst, int32_t* tokens_dst,
                  int32_t* src_of_dst, int64_t* n_pages_used,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * arrol_compact for callers that cannot allocate or pass scratch memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same operation with the same arguments,
 * outputs and error rules as arrol_compact, minus the workspace.  The per-survivor base offsets live in
 * a fixed device array inside the library (ARROL_COMPACT_STATIC_MAX_KEEP + 1 int32 = 64 KiB, held by
 * every GPU the library runs on until the process ends); the call allocates and frees nothing.
 * n_keep > ARROL_COMPACT_STATIC_MAX_KEEP returns ARROL_EWORKSPACE with nothing enqueued; ARROL_EHIP if
 * the array's device address cannot be obtained (looked up once per device, on the first call there).
 * All calls on one GPU share that array: two calls whose kernels may overlap on the same GPU (different
 * streams, or several host threads) race - serialise them, or use arrol_compact with separate workspaces.
 */
#define ARROL_COMPACT_STATIC_MAX_KEEP 16383
int arrol_compact_static(const void* kv_src, arrol_kv_layout src, void* kv_dst, arrol_kv_layout dst,
                         const int32_t* block_table_src, const int32_t* seq_len_src,
                         int32_t max_pages_per_seq, const int32_t* tokens_src, int32_t max_len,
                         const int32_t* survivor_idx, int32_t n_src, int32_t n_keep,
                         int32_t* block_table_dst, int32_t* seq_len_dst, int32_t* tokens_dst,
                         int32_t* src_of_dst, int64_t* n_pages_used, void* stream);

/*
 * Stage 3, in-place variant ("hole filling").  Same paper passage: pruned requests leave the pool so that
 * the freed capacity is re-used (Sec. 4.3 (i)); no second pool is needed and only the pages that lie in the
 * wrong place move.  With live = the set of physical pages the survivors reference (first
 * ceil(seq_len/page_tokens) table entries each) and n_live its size: holes = pages < n_live that are not
 * live, movers = live pages >= n_live, both ascending; page movers[k] is copied (every layer, K and V) onto
 * page holes[k], all other pages stay untouched.  Afterwards the survivors occupy exactly pages
 * [0, n_live) of the SAME pool and [n_live, n_pages) is free.
 *   block_table_dst[r][p] = final page of survivor rank r's logical page p, -1 beyond its length;
 *   seq_len_dst[r], src_of_dst[r] as in arrol_compact; *n_pages_used = n_live; *n_moved (NULL allowed) =
 *   number of pages copied.
 * A survivor id outside [0, n_src) is an empty rollout; table entries outside [0, n_pages) are ignored
 * (reported as -1).  Token buffers are not touched (they are indexed by rollout, not by page).
 * workspace: arrol_compact_inplace_workspace_bytes(layout.n_pages) bytes, 16-byte aligned.
 */
size_t arrol_compact_inplace_workspace_bytes(int64_t n_pages);
int arrol_compact_inplace(void* kv, arrol_kv_layout layout, const int32_t* block_table_src,
                          const int32_t* seq_len_src, int32_t max_pages_per_seq,
                          const int32_t* survivor_idx, int32_t n_src, int32_t n_keep,
                          int32_t* block_table_dst, int32_t* seq_len_dst, int32_t* src_of_dst,
                          int64_t* n_pages_used, int64_t* n_moved, void* workspace,
                          size_t workspace_bytes, void* stream);

/*
 * Stage 4 -- per-token log-probability of the sampled token (the policy term of GRPO's
 * importance ratio, Sec. 3; computed on the re-batched survivors, Sec. 4.3 (ii), Alg. 1):
 *   z_t = W h_t,  logprob_t = z_t[y_t] - logsumexp_v z_t[v]      (temperature 1, no bias)
 * hidden   bf16 [T, d] packed rows (ragged survivors concatenated), 16-byte aligned.
 * lm_head  bf16 [V, d] row-major, 16-byte aligned.   d multiple of 8, d >= 8; V >= 1.
 * targets  int32 [T]; a target outside [0, V) yields NaN in logprob_out for that row.
 * logprob_out fp32 [T];  lse_out NULL or fp32 [T] (the logsumexp).
 * bf16 products accumulated in fp32 on the matrix cores; the [T, V] logits are never
 * written to memory.  T == 0 is a no-op.
 * n_splits  number of ranges the vocabulary is cut into (each workgroup walks one range for its block of
 *           tokens; the per-range partials are merged by a second small kernel).  0 lets the library
 *           choose from T and V; a positive value is used as given, capped at the number of 256-row
 *           vocabulary tiles.  The result does not depend on it beyond fp32 rounding of the merge.
 * workspace: arrol_logprob_workspace_bytes(T, V, d, n_splits) bytes for the SAME n_splits, 16-byte aligned.
 */
size_t arrol_logprob_workspace_bytes(int64_t T, int32_t V, int32_t d, int32_t n_splits);
int arrol_logprob(const void* hidden, const void* lm_head, const int32_t* targets,
                  int64_t T, int32_t V, int32_t d, float* logprob_out, float* lse_out,
                  int32_t n_splits, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Stage 5 -- rank-weighted vote (Sec. 4.4: candidates are sorted by head score and their
 * ranks rescaled linearly to [0,1]; the weights replace the unit votes of a majority vote).
 * Per question with candidates i < C:
 *   rank2_i = 2*#{j: q_j < q_i} + #{j != i: q_j == q_i}   (twice the average rank; weight = rank2/(2(C-1)))
 *   tally[a] = sum of rank2_i over candidates with answer a
 *   winner   = answer id with the largest tally among ids that occur, lowest id on ties
 * prob       fp32 [n_questions*C] (any monotone score; finite)
 * answer_id  int32 [n_questions*C]; ids outside [0, n_answers) take no part (a question
 *            whose ids are all outside gets winner -1).
 * winner     int32 [n_questions];  tally NULL or int64 [n_questions, n_answers].
 * Requires 1 <= C <= ARROL_MAX_GROUP, n_answers >= 1.
 */
int arrol_weighted_vote(const float* prob, const int32_t* answer_id, int32_t n_questions,
                        int32_t C, int32_t n_answers, int32_t* winner, int64_t* tally,
                        void* stream);

/*
 * ---- The paper's practical (stochastic) pruning policy: App. A.4, Eq. 1-2; Alg. 1 backend --------------
 * The frontend turns its labelled score buffers into histogram parameters; the backend looks up a
 * survival probability for each rollout that reaches the detection length and prunes it with
 * probability 1 - p.  Unlike arrol_select the number of survivors is random (kappa*N in expectation).
 */
#define ARROL_MAX_BINS 2048

/*
 * App. A.4 Eq. 1: c_b^+ = #{k : label_k = 1, b(s_k) = b},  c_b^- likewise for label 0, with the uniform
 * bin b(s') = min(B-1, floor(B*s')) (product in fp32) of the sigmoid-normalised score s' in [0,1].
 * s_norm fp32 [M], label uint8 [M] (0 / non-zero), c_pos / c_neg int64 [B] are OVERWRITTEN.
 * 1 <= B <= ARROL_MAX_BINS.  M == 0 zeroes the counts.
 */
int arrol_histogram(const float* s_norm, const uint8_t* label, int64_t M, int32_t B,
                    int64_t* c_pos, int64_t* c_neg, void* stream);

typedef struct arrol_policy {
    float kappa;   /* target keep rate                    (paper: 0.5) */
    float rho;     /* target positive ratio               (paper: 0.5) */
    float lambda;  /* strength of the balance correction  (paper: 0.5) */
    float p_min;   /* clip range of the survival probability (not given in the paper) */
    float p_max;
    float alpha;   /* Laplace smoothing of the histograms    (not given in the paper) */
} arrol_policy;

/*
 * App. A.4: Laplace-smoothed likelihoods P(b|Y) = (c_b + alpha) / (sum c + alpha*B), prior pi = N+/(N+ + N-)
 * (1/2 for empty buffers), Bayes posterior q(b) = pi P(b|1) / (pi P(b|1) + (1-pi) P(b|0)); Eq. 2:
 * p(b) = clip(kappa + delta + lambda (rho - q(b)), p_min, p_max), with delta found by 64 bisection steps on
 * [p_min - kappa - lambda, p_max - kappa + lambda] so that sum_b w_b p(b) = kappa, w_b = (c_b^+ + c_b^-)/total
 * (the buffer distribution; uniform for empty buffers).  Computed in fp64.
 * q_lut, p_lut fp32 [B]; delta NULL or a device double.  Policy fields must satisfy 0 <= kappa, rho <= 1,
 * lambda >= 0, 0 <= p_min <= p_max <= 1, alpha >= 0.
 */
int arrol_calibrate(const int64_t* c_pos, const int64_t* c_neg, int32_t B, arrol_policy pol,
                    float* q_lut, float* p_lut, double* delta, void* stream);

/*
 * Alg. 1, backend: a rollout that reaches the detection length is pruned with probability 1 - p_i and the
 * decision recorded.  p_i = p_lut[b(s_i)], rollout i survives iff
 * uniforms[i] < p_i (fp32 comparison; the caller supplies the random numbers).
 * s_norm, uniforms fp32 [N]; p_lut fp32 [B]; p_out NULL or fp32 [N]; keep_mask uint8 [N];
 * survivor_idx int32 [N]: the survivors' ids ascending, then -1 up to N (so it can be handed to
 * arrol_compact with n_keep = N: entries -1 yield empty destination rollouts); n_survivors device int32.
 */
int arrol_prune_bernoulli(const float* s_norm, const float* uniforms, int32_t N, const float* p_lut,
                          int32_t B, float* p_out, uint8_t* keep_mask, int32_t* survivor_idx,
                          int32_t* n_survivors, void* stream);

/*
 * ---- Trace confidence (Sec. 3 "Trace Confidence": the model-intrinsic signal the quality head is compared
 * with, and the voting weight of the DeepConf-style test-time baseline) ---------------------------------------
 * Token confidence  H_t = - sum_{j=1..V} log P_t(j)  with P_t = softmax(W h_t)
 *                       = V * lse_t - <h_t, sum_j W_j>,
 * lse_t being the logsumexp arrol_logprob already returns, so no second [T, V] product is formed.
 * hidden, lm_head, T, V, d as in arrol_logprob (d <= 16384); lse fp32 [T] (arrol_logprob's lse_out for the
 * same hidden and lm_head); conf_out fp32 [T].  A NaN in lse propagates.  T == 0 is a no-op.
 * workspace: arrol_token_confidence_workspace_bytes(V, d) bytes, 16-byte aligned.
 */
size_t arrol_token_confidence_workspace_bytes(int32_t V, int32_t d);
int arrol_token_confidence(const void* hidden, const void* lm_head, const float* lse, int64_t T,
                           int32_t V, int32_t d, float* conf_out, void* workspace,
                           size_t workspace_bytes, void* stream);

/*
 * Trace-level aggregates of the token confidences (Sec. 3).  Trace i is tokens [cu_seqlens[i],
 * cu_seqlens[i+1]) of conf (offsets are clamped into [0, T]); with L its length and w = min(window, L):
 *   mean_out[i]    average token confidence over the trace (the self-uncertainty score),
 *   windows        H_w = mean of w consecutive tokens, one window per start position (L - w + 1 of them),
 *   min_out[i]     the smallest window value,
 *   bottom_out[i]  mean of the lowest max(1, ceil(bottom_percent * n_windows / 100)) window values.
 * conf fp32 [T]; cu_seqlens int64 [n_seq+1]; outputs fp64 [n_seq], NaN for an empty trace; fp64 arithmetic.
 * window >= 1, 1 <= bottom_percent <= 100 (the paper's "bottom 10 %" is 10), else ARROL_EINVAL.
 * workspace: arrol_trace_confidence_workspace_bytes(T, n_seq) bytes, 16-byte aligned.  n_seq == 0 is a no-op.
 */
size_t arrol_trace_confidence_workspace_bytes(int64_t T, int32_t n_seq);
int arrol_trace_confidence(const float* conf, const int64_t* cu_seqlens, int64_t T, int32_t n_seq,
                           int32_t window, int32_t bottom_percent, double* mean_out, double* min_out,
                           double* bottom_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * ---- GRPO on the survivors (Sec. 3 "Group-Relative Policy Optimization"; Alg. 1, advantage step) -------------
 * Group-relative advantage  A_i = (R_i - mean(R_group)) / (std(R_group) + eps)  over the rollouts of one prompt
 * that survived pruning; rollouts of group g are [group_offsets[g], group_offsets[g+1]) (int64 [n_groups+1],
 * clamped into [0, N]).  std^2 = sum (R - mean)^2 / (n - ddof), ddof 0 (population) or 1; std = 0 when
 * n - ddof <= 0; A_i = 0 where std + eps == 0 (all rewards equal).  fp64 arithmetic, fp32 results.
 * reward fp32 [N]; advantage fp32 [N]; seq_weight NULL or fp32 [N] = 1 / (group size * n_groups), the weight
 * of rollout i in the objective below.  Rollouts outside every group are not written.
 */
int arrol_grpo_advantage(const float* reward, const int64_t* group_offsets, int64_t N, int32_t n_groups,
                         int32_t ddof, float eps, float* advantage, float* seq_weight, void* stream);

/*
 * Clipped-ratio objective of Sec. 3 on packed per-token log-probabilities (rollout i = tokens
 * [cu_seqlens[i], cu_seqlens[i+1])):
 *   J = sum_i seq_weight_i * (1/|o_i|) * sum_t [ min(r_t A_i, clip(r_t, 1-eps_low, 1+eps_high) A_i) - beta*kl_t ]
 *   r_t = exp(logp_t - logp_ref_t),  kl_t = exp(u) - u - 1 with u = logp_ref_t - logp_t
 * (the paper writes beta*KL(pi_theta || pi_ref) without an estimator; kl_t is non-negative and its mean under
 * pi_theta is that divergence).  With seq_weight from arrol_grpo_advantage this is the mean over groups of the
 * mean over the group's rollouts of the per-token mean.  An empty rollout adds 0.
 * logp, logp_ref fp32 [T]; advantage, seq_weight fp32 [n_seq]; objective_out NULL or fp64 [1];
 * grad_logp NULL or fp32 [T] = dJ/dlogp_t (zero where the clipped branch is the minimum); n_clipped NULL or
 * int64 [1] = tokens where the clipped branch is strictly smaller.  fp64 arithmetic, fixed summation order.
 * 0 <= eps_low <= 1, eps_high >= 0, beta >= 0, else ARROL_EINVAL.  n_seq == 0 writes J = 0.
 * workspace: arrol_grpo_objective_workspace_bytes(n_seq) bytes, 16-byte aligned.
 */
size_t arrol_grpo_objective_workspace_bytes(int32_t n_seq);
int arrol_grpo_objective(const float* logp, const float* logp_ref, const int64_t* cu_seqlens, int64_t T,
                         int32_t n_seq, const float* advantage, const float* seq_weight, float eps_low,
                         float eps_high, float beta, double* objective_out, float* grad_logp,
                         int64_t* n_clipped, void* workspace, size_t workspace_bytes, void* stream);

/*
 * ---- Training the quality head (Sec. 4.2; Sec. 4.3 (iii); Alg. 1, the frontend's optimizer step) ----
 * The head is fitted on the fly to the rollouts' final rewards with a cross-entropy loss; the hidden states
 * are constants (no gradient reaches the backbone).  For the linear head, with q_i = sigmoid(<w,h_i> + bias):
 *   L = -(1/N) sum_i [ y_i log q_i + (1-y_i) log(1-q_i) ]
 *   dL/dw = (1/N) sum_i (q_i - y_i) h_i,   dL/dbias = (1/N) sum_i (q_i - y_i)
 * hidden, row_stride_elems, row_index, w, bias as in arrol_score; labels fp32 [n_rows] in [0,1] (the reward
 * of output row i).  8 <= d <= 8192, d a multiple of 8.
 * loss_out NULL or fp32 [1]; grad_w fp32 [d]; grad_bias NULL or fp32 [1].  fp32 arithmetic, sums in a fixed
 * order (bit-reproducible run to run).  n_rows == 0 writes zeros.
 * workspace: device memory of at least arrol_score_grad_workspace_bytes(n_rows, d), caller-owned, contents
 * undefined afterwards; too small or NULL -> ARROL_EWORKSPACE.
 */
size_t arrol_score_grad_workspace_bytes(int32_t n_rows, int32_t d);
int arrol_score_grad(const void* hidden, int64_t row_stride_elems, const int64_t* row_index,
                     const float* w, float bias, const float* labels, int32_t n_rows, int32_t d,
                     float* loss_out, float* grad_w, float* grad_bias, void* workspace,
                     size_t workspace_bytes, void* stream);

/*
 * The same loss for the MLP head of arrol_score_mlp (a = relu(W1 h + b1), s = <w2,a> + b2), with the
 * gradient of every head parameter.  With r_i = (q_i - y_i)/N and delta_i = r_i * w2 * [W1 h_i + b1 > 0]:
 *   dL/db2 = sum_i r_i,  dL/dw2 = sum_i r_i a_i,  dL/db1 = sum_i delta_i,  dL/dW1 = sum_i delta_i h_i^T
 * hidden, row_stride_elems, row_index, w1, b1, w2, b2, n_rows, d, m as in arrol_score_mlp; labels fp32 [n_rows].
 * loss_out NULL or fp32 [1]; grad_w1 fp32 [m, d]; grad_b1, grad_w2 fp32 [m]; grad_b2 NULL or fp32 [1].
 * delta is rounded to bf16 before the contraction over the rollouts (bf16 products, fp32 accumulation);
 * everything else is fp32; sums in a fixed order (bit-reproducible run to run).
 * delta_terms: 1 = delta as one bf16 value (relative rounding 2^-9 per term of dL/dW1); 2 = delta as the sum
 * of two bf16 values, hi = bf16(delta) and lo = bf16(delta - hi), contracted one after the other (relative
 * rounding 2^-17: dL/dW1 to fp32 accuracy, at twice the cost of that contraction).  Other values -> ARROL_EINVAL.
 * n_rows == 0 writes zeros.
 * workspace: arrol_score_mlp_grad_workspace_bytes(n_rows, d, m, delta_terms) bytes, 256-byte aligned,
 * caller-owned, contents undefined afterwards; too small or NULL -> ARROL_EWORKSPACE.
 */
size_t arrol_score_mlp_grad_workspace_bytes(int32_t n_rows, int32_t d, int32_t m, int32_t delta_terms);
int arrol_score_mlp_grad(const void* hidden, int64_t row_stride_elems, const int64_t* row_index,
                         const void* w1, const float* b1, const float* w2, float b2, const float* labels,
                         int32_t n_rows, int32_t d, int32_t m, float* loss_out, float* grad_w1,
                         float* grad_b1, float* grad_w2, float* grad_b2, int32_t delta_terms,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * One AdamW update in place (the paper names no optimizer; AdamW with decoupled weight decay is this
 * build's reading).  With t = step >= 1:
 *   m <- beta1 m + (1-beta1) g;  v <- beta2 v + (1-beta2) g^2
 *   p <- p - lr * ( (m/(1-beta1^t)) / (sqrt(v/(1-beta2^t)) + eps) + weight_decay * p )
 * param, m, v fp32 [n] updated in place; grad fp32 [n]; all device pointers.  param_bf16: NULL, or bf16 [n]
 * that receives the updated parameters rounded to nearest even (the copy arrol_score_mlp reads).
 * 0 <= beta1, beta2 < 1, eps >= 0, else ARROL_EINVAL.  n == 0 is a no-op.
 */
int arrol_adamw_step(float* param, const float* grad, float* m, float* v, int64_t n, int32_t step,
                     float lr, float beta1, float beta2, float eps, float weight_decay,
                     void* param_bf16, void* stream);

/*
 * Measurement aid for the benchmark, not a stage of the path (the paper defines no such call): runs bf16
 * MFMAs from registers alone - no LDS, no memory traffic in the loop, 8 wavefronts per workgroup, the
 * accumulator shape of the log-prob kernel - and so shows what this card's matrix cores sustain on the given
 * operand VALUES: the part lowers its clock under a power limit when operands toggle, not when they are zero.
 * a_bf16 [n_a], b_bf16 [n_b]: device, bf16, 16-byte aligned, n_a and n_b positive multiples of 512 (whole
 * 64-lane fragments); each wavefront takes 8 A and 4 B fragments round-robin from them, once, before the loop.
 * shape: 16 -> v_mfma_f32_16x16x32_bf16 (32 instructions per iteration), 32 -> v_mfma_f32_32x32x16_bf16 (16).
 * n_workgroups in [1, 65536] workgroups of 512 lanes; iters >= 0 loop iterations of 524,288 flop per wavefront.
 * sink: device fp32 [n_workgroups * 512], receives each lane's sum of its accumulators (iters * the lane's share
 * of A B^T, fp32 accumulation order fixed).  flop_out: host double or NULL, receives the launch's flop count.
 * Asynchronous on `stream`; time it with events.  Anything else -> ARROL_EINVAL, nothing enqueued.
 */
int arrol_probe_mfma_rate(const void* a_bf16, int64_t n_a, const void* b_bf16, int64_t n_b, int32_t shape,
                          int32_t n_workgroups, int32_t iters, float* sink, double* flop_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ARROL_H */
