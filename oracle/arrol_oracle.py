"""CPU oracle for the ARRoL online rollout-pruning data path.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, obviously
correct restatement of what each stage computes, written from the paper
("Prune as You Generate: Online Rollout Pruning for Faster and Better RLVR").
Floating point is float64 on the exact values of the bf16 / fp32 inputs;
integer stages use unbounded Python integers.  It shares no code with the HIP
library and must never be imported by it.  Only the test-suite, the smoke
check and the benchmark's cpu_baseline leg may call it.

Every function is pinned by CPU tests to facts the paper and the mathematics
fix (closed forms, invariants, brute force in exact rationals); none is
"parity unpinned".

Stages (paper passages in each docstring):
  score          quality head + sigmoid            Sec. 4.2, App. A.4
  select         balance rule iterated G-K times   Sec. 4.1 Thm 4.2, App. A.1
  compact        survivor gather / re-batch        Sec. 4.3 (i),(ii); Alg. 1
  logprob        log pi(o_t | o_<t)                Sec. 3 (GRPO ratio); Alg. 1
  weighted_vote  rank-weighted answer vote         Sec. 4.4
  histogram / calibrate / prune_bernoulli   the practical policy   App. A.4 Eq. 1-2; Alg. 1
  score_mlp, score_ce(_grad), adamw_step    quality head variants and training   Sec. 4.2, 4.3 (iii)
  token_confidence / trace_confidence       trace confidence   Sec. 3
  grpo_advantage / grpo_objective           group-relative advantage, clipped objective   Sec. 3
"""
import math

import numpy as np

FIXED_POINT_BITS = 30  # probabilities are read on a 2**-30 grid by select()


# ----------------------------------------------------------------------------
# helpers: exact widening of bf16 bit patterns
# ----------------------------------------------------------------------------
def bf16_bits_to_f64(bits):
    """uint16 bf16 bit patterns -> float64, exactly (bf16 is the top half of
    an IEEE binary32)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


# ----------------------------------------------------------------------------
# stage 1: score
# ----------------------------------------------------------------------------
def score(hidden_bits, w, bias=0.0):
    """Quality-head score and its sigmoid.

    Sec. 4.2 ("Quality Score Prediction"): a small head on the backbone's
    hidden state gives a scalar s_i per partial rollout.  App. A.4: the score
    is squashed into [0,1] with the sigmoid.  Reading used here: the head is
    one linear layer, s_i = <w, h_i> + b, and the squashed score is the
    success probability q_i handed to the selection stage.

    hidden_bits : [N, d] uint16 (bf16 bit patterns)
    w           : [d] float32, bias: float
    returns (s, q) float64 [N]
    """
    h = bf16_bits_to_f64(hidden_bits)
    w64 = np.asarray(w, dtype=np.float32).astype(np.float64)
    n = h.shape[0]
    s = np.empty(n, dtype=np.float64)
    for i in range(n):
        s[i] = math.fsum(h[i] * w64) + float(bias)
    q = np.empty(n, dtype=np.float64)
    for i in range(n):
        if s[i] >= 0.0:
            q[i] = 1.0 / (1.0 + math.exp(-s[i]))
        else:  # same function, written so exp never overflows
            e = math.exp(s[i])
            q[i] = e / (1.0 + e)
    return s, q


# ----------------------------------------------------------------------------
# stage 2: select
# ----------------------------------------------------------------------------
def quantise(prob_f32):
    """fp32 probabilities -> integers on the 2**-30 grid, rounding the fp32
    product to nearest-even *in fp32* (the product by a power of two is exact,
    so this is a pure rounding of the given value).  Both the oracle and the
    library take the selection decision on these integers."""
    p = np.asarray(prob_f32, dtype=np.float32)
    scaled = p * np.float32(2.0 ** FIXED_POINT_BITS)      # exact in fp32
    return [int(v) for v in np.rint(scaled).astype(np.int64)]


def select_group(k, K, R):
    """One prompt group.  k: list of G fixed-point probabilities, R: fixed-point
    target ratio rho.  Sec. 4.1, Thm 4.2 / App. A.1: with live set A,
        mu_{-j} = (1/(|A|-1)) * sum_{i in A, i != j} q_i
        j_hat   = argmin_{j in A} | mu_{-j} - rho |
    and j_hat is pruned.  The rule is applied again to the shrunken group until
    K rollouts remain.  Ties in the argmin go to the lowest index.

    |mu_{-j} - rho| is compared over a common denominator (|A|-1) * 2**30, so
    everything below is exact integer arithmetic on the definition itself.
    Returns (survivors ascending, removal order)."""
    live = list(range(len(k)))
    removed = []
    while len(live) > K:
        n = len(live)
        best_j, best_dev = None, None
        for j in live:
            rest = sum(k[i] for i in live if i != j)       # (n-1) * mu_{-j} * 2^30
            dev = abs(rest - R * (n - 1))                  # (n-1) * |mu_{-j}-rho| * 2^30
            if best_dev is None or dev < best_dev:
                best_j, best_dev = j, dev
        live.remove(best_j)
        removed.append(best_j)
    return live, removed


def select(prob_f32, n_groups, G, K, rho=0.5):
    """Exactly-K, correctness-balanced survivors for every prompt group.

    prob_f32: [n_groups*G] float32, groups are consecutive runs of G rollouts.
    Returns keep_mask uint8 [n_groups*G] and survivor_idx int32 [n_groups*K]
    (global rollout ids, ascending within a group, groups in order)."""
    if not (1 <= K <= G):
        raise ValueError("need 1 <= K <= G")
    k_all = quantise(prob_f32)
    if len(k_all) != n_groups * G:
        raise ValueError("prob has wrong length")
    R = quantise(np.array([rho], dtype=np.float32))[0]
    keep = np.zeros(n_groups * G, dtype=np.uint8)
    surv = np.empty(n_groups * K, dtype=np.int32)
    for g in range(n_groups):
        live, _ = select_group(k_all[g * G:(g + 1) * G], K, R)
        for r, j in enumerate(live):
            keep[g * G + j] = 1
            surv[g * K + r] = g * G + j
    return keep, surv


# ----------------------------------------------------------------------------
# stage 3: compact
# ----------------------------------------------------------------------------
def compact(kv_src, block_table_src, seq_len_src, tokens_src, survivor_idx,
            n_pages_dst, fill=0):
    """Gather the survivors' paged KV cache and token buffers into a dense pool.

    Sec. 4.3 (i): pruned requests leave the pool at once so their capacity is
    reused; (ii) / Alg. 1's frontend step that drops pruned rollouts: survivors are
    re-batched.  The paper fixes no layout; this build's contract is:

    kv_src          [L, 2, P_src, page_tokens, H_kv, hd] uint16 (bf16 bits)
    block_table_src [N, ppr] int32, seq_len_src [N] int32, tokens_src [N, max_len] int32
    survivor_idx    [N_k] int32, ascending rollout ids
    Survivor rank r owns np_r = ceil(seq_len/page_tokens) destination pages
    starting at base_r = sum_{r'<r} np_r'; whole pages are copied verbatim.

    Returns dict(kv_dst, block_table_dst, seq_len_dst, tokens_dst, src_of_dst,
    n_pages_used).  Untouched destination pages hold `fill`."""
    L, two, _, page_tokens, H, hd = kv_src.shape
    assert two == 2
    n_keep = len(survivor_idx)
    ppr = block_table_src.shape[1]
    kv_dst = np.full((L, 2, n_pages_dst, page_tokens, H, hd), fill, dtype=kv_src.dtype)
    bt_dst = np.full((n_keep, ppr), -1, dtype=np.int32)
    sl_dst = np.empty(n_keep, dtype=np.int32)
    tok_dst = np.empty((n_keep, tokens_src.shape[1]), dtype=np.int32)
    src_of_dst = np.empty(n_keep, dtype=np.int32)
    base = 0
    for r in range(n_keep):
        src = int(survivor_idx[r])
        n_pages = -(-int(seq_len_src[src]) // page_tokens)
        for p in range(n_pages):
            sp = int(block_table_src[src, p])
            for layer in range(L):
                for c in range(2):
                    kv_dst[layer, c, base + p] = kv_src[layer, c, sp]
            bt_dst[r, p] = base + p
        sl_dst[r] = seq_len_src[src]
        tok_dst[r, :] = tokens_src[src, :]
        src_of_dst[r] = src
        base += n_pages
    return dict(kv_dst=kv_dst, block_table_dst=bt_dst, seq_len_dst=sl_dst,
                tokens_dst=tok_dst, src_of_dst=src_of_dst, n_pages_used=base)


# ----------------------------------------------------------------------------
# stage 4: logprob
# ----------------------------------------------------------------------------
def log_softmax_rows(hidden_bits, lm_head_bits):
    """Full float64 log-softmax over the vocabulary for every row:
    z = W h, log_softmax(z)_v = z_v - (m + log sum_v exp(z_v - m)), m = max z."""
    h = bf16_bits_to_f64(hidden_bits)
    W = bf16_bits_to_f64(lm_head_bits)
    z = h @ W.T
    m = z.max(axis=1, keepdims=True)
    lse = m + np.log(np.exp(z - m).sum(axis=1, keepdims=True))
    return z - lse, lse[:, 0]


def logprob(hidden_bits, lm_head_bits, targets):
    """Per-token log-probability of the sampled token under the policy,
    log pi_theta(o_t | o_<t): the quantity inside GRPO's importance ratio
    (Sec. 3) that the frontend computes on the re-batched survivors (Sec. 4.3
    (ii); Alg. 1's frontend step for rewards and log-probs).  Temperature 1, no LM-head
    bias; row t of `hidden` is already aligned with targets[t].

    hidden_bits [T, d] uint16, lm_head_bits [V, d] uint16, targets [T] int.
    Returns (logp, lse) float64 [T].  Rows are processed in small batches only
    to bound memory; each row's arithmetic is the definition above."""
    T = hidden_bits.shape[0]
    targets = np.asarray(targets, dtype=np.int64)
    W = bf16_bits_to_f64(lm_head_bits)
    logp = np.empty(T, dtype=np.float64)
    lse = np.empty(T, dtype=np.float64)
    step = max(1, min(T, (1 << 25) // max(1, W.shape[0])))
    for t0 in range(0, T, step):
        h = bf16_bits_to_f64(hidden_bits[t0:t0 + step])
        z = h @ W.T
        m = z.max(axis=1)
        l = m + np.log(np.exp(z - m[:, None]).sum(axis=1))
        lse[t0:t0 + step] = l
        logp[t0:t0 + step] = z[np.arange(z.shape[0]), targets[t0:t0 + step]] - l
    return logp, lse


# ----------------------------------------------------------------------------
# stage 5: weighted vote
# ----------------------------------------------------------------------------
def weighted_vote(prob_f32, answer_id, n_questions, C, A):
    """Rank-weighted vote (Sec. 4.4): candidates are sorted by head score and
    their ranks rescaled linearly to [0,1]; the answer with the largest summed
    weight wins.  Readings: higher score = higher rank; equal scores share the
    average of their ranks; ranks are kept as integers by doubling
    (rank2_i = 2*#{q_j < q_i} + #{j != i: q_j == q_i}, weight = rank2/(2(C-1)));
    the argmax runs over answer ids that occur among the candidates, lowest id
    on equal tallies.

    Returns winner int32 [Q], tally int64 [Q, A] in rank2 units."""
    q = np.asarray(prob_f32, dtype=np.float32).reshape(n_questions, C)
    ans = np.asarray(answer_id, dtype=np.int64).reshape(n_questions, C)
    winner = np.empty(n_questions, dtype=np.int32)
    tally = np.zeros((n_questions, A), dtype=np.int64)
    for u in range(n_questions):
        rank2 = []
        for i in range(C):
            below = sum(1 for j in range(C) if q[u, j] < q[u, i])
            equal = sum(1 for j in range(C) if j != i and q[u, j] == q[u, i])
            rank2.append(2 * below + equal)
        for i in range(C):
            tally[u, ans[u, i]] += rank2[i]
        best = None
        for a in sorted(set(int(x) for x in ans[u])):
            if best is None or tally[u, a] > tally[u, best]:
                best = a
        winner[u] = best
    return winner, tally


# ----------------------------------------------------------------------------
# the paper's practical pruning policy (App. A.4; Alg. 1 backend lines)
# ----------------------------------------------------------------------------
def bin_index(s_norm_f32, B):
    """Uniform bin of a normalised score, b(s') = min(B-1, floor(B * s')) (App. A.4).  The product is
    taken in fp32 (exact for B a power of two), which is where both sides take the decision."""
    s = np.asarray(s_norm_f32, dtype=np.float32)
    b = np.floor(s * np.float32(B)).astype(np.int64)
    return np.minimum(B - 1, np.maximum(0, b))


def histogram(s_norm_f32, label, B):
    """Histogram counts of the two labelled buffers (App. A.4 Eq. 1):
    c_b^+ = #{k : b(s_k^+) = b},  c_b^- = #{k : b(s_k^-) = b}."""
    b = bin_index(s_norm_f32, B)
    lab = np.asarray(label).astype(bool)
    c_pos = np.zeros(B, dtype=np.int64)
    c_neg = np.zeros(B, dtype=np.int64)
    for k in range(len(b)):
        if lab[k]:
            c_pos[b[k]] += 1
        else:
            c_neg[b[k]] += 1
    return c_pos, c_neg


def posterior_lut(c_pos, c_neg, alpha):
    """Binned posterior q(b) = P(Y=1 | b) by Bayes' rule with Laplace-smoothed likelihoods (App. A.4):
        P(b|Y=1) = (c_b^+ + alpha) / (sum_b' c_b'^+ + alpha B),  same for Y=0,
        q(b) = pi P(b|1) / (pi P(b|1) + (1-pi) P(b|0)),  pi = P(Y=1) estimated from the buffers.
    Reading: pi = N^+ / (N^+ + N^-), 1/2 when both buffers are empty."""
    c_pos = np.asarray(c_pos, dtype=np.float64)
    c_neg = np.asarray(c_neg, dtype=np.float64)
    B = len(c_pos)
    n_pos, n_neg = c_pos.sum(), c_neg.sum()
    pi = 0.5 if n_pos + n_neg == 0 else n_pos / (n_pos + n_neg)
    like_pos = (c_pos + alpha) / (n_pos + alpha * B)
    like_neg = (c_neg + alpha) / (n_neg + alpha * B)
    num = pi * like_pos
    den = num + (1.0 - pi) * like_neg
    q = np.where(den > 0, num / np.where(den > 0, den, 1.0), pi)
    return q, pi


def bin_weights(c_pos, c_neg):
    """The buffer distribution over bins used for the expectation E[p]: w_b = (c_b^+ + c_b^-)/total,
    uniform when the buffers are empty."""
    tot = np.asarray(c_pos, dtype=np.float64) + np.asarray(c_neg, dtype=np.float64)
    s = tot.sum()
    return tot / s if s > 0 else np.full(len(tot), 1.0 / len(tot))


def survival_lut(q, w, kappa, rho, lam, p_min, p_max, iters=64):
    """Survival probability per bin (App. A.4 Eq. 2): p = clip(kappa + delta + lambda (rho - q), p_min, p_max),
    with the scalar delta found by binary search so that the expected keep rate under the buffer
    distribution matches kappa: sum_b w_b p_b = kappa.  Reading: the bracket is
    [p_min - kappa - lambda, p_max - kappa + lambda] (every bin clipped low / high at its ends), `iters`
    halvings, delta = the final midpoint."""
    q = np.asarray(q, dtype=np.float64)

    def p_of(delta):
        return np.clip(kappa + delta + lam * (rho - q), p_min, p_max)

    lo, hi = p_min - kappa - lam, p_max - kappa + lam
    for _ in range(iters):
        mid = 0.5 * (lo + hi)
        if float(np.dot(w, p_of(mid))) < kappa:
            lo = mid
        else:
            hi = mid
    delta = 0.5 * (lo + hi)
    return p_of(delta), delta


def calibrate(c_pos, c_neg, kappa, rho, lam, p_min, p_max, alpha):
    """Histogram parameters h_t the frontend sends to the backend (Alg. 1): per-bin posterior q, per-bin
    survival probability p and the bias delta."""
    q, _ = posterior_lut(c_pos, c_neg, alpha)
    p, delta = survival_lut(q, bin_weights(c_pos, c_neg), kappa, rho, lam, p_min, p_max)
    return q, p, delta


def prune_bernoulli(s_norm_f32, uniforms_f32, p_lut_f32):
    """Backend decision when a rollout first reaches the detection length (Alg. 1): look up its survival
    probability p_i by the bin of its normalised score and prune it with probability 1 - p_i.  The random
    numbers are passed in: rollout i survives iff u_i < p_i (both fp32).  Returns p [N] fp32,
    keep_mask uint8 [N], survivor_idx int32 (ascending), n_survivors."""
    p_lut = np.asarray(p_lut_f32, dtype=np.float32)
    b = bin_index(s_norm_f32, len(p_lut))
    p = p_lut[b]
    u = np.asarray(uniforms_f32, dtype=np.float32)
    keep = np.zeros(len(u), dtype=np.uint8)
    surv = []
    for i in range(len(u)):
        if u[i] < p[i]:
            keep[i] = 1
            surv.append(i)
    return p, keep, np.asarray(surv, dtype=np.int32), len(surv)


# ----------------------------------------------------------------------------
# in-place compaction ("hole filling") of the paged KV pool
# ----------------------------------------------------------------------------
def compact_inplace(kv, block_table_src, seq_len_src, survivor_idx):
    """Sec. 4.3 (i): pruned requests leave the pool at once so that the freed capacity can be re-used.
    The paper fixes no mechanism; this build's in-place contract: after the call the survivors' pages
    occupy the dense prefix [0, n_live) of the SAME pool, moving as few pages as possible:
      live   = set of physical pages referenced by the survivors (first ceil(seq_len/page_tokens) entries)
      holes  = pages < n_live that are not live, ascending;  movers = live pages >= n_live, ascending
      page movers[k] is copied (every layer, K and V) onto holes[k]; all other pages are untouched.
    kv is modified in place.  Returns dict(block_table_dst [N_k, ppr] with -1 padding, seq_len_dst,
    src_of_dst, n_pages_used = n_live, n_moved)."""
    L, two, P, page_tokens, H, hd = kv.shape
    ppr = block_table_src.shape[1]
    n_keep = len(survivor_idx)
    live = set()
    pages_of = []
    for r in range(n_keep):
        s = int(survivor_idx[r])
        n_pages = -(-int(seq_len_src[s]) // page_tokens) if s >= 0 else 0
        row = [int(block_table_src[s, p]) for p in range(n_pages)]
        pages_of.append(row)
        live.update(row)
    n_live = len(live)
    holes = [p for p in range(n_live) if p not in live]
    movers = sorted(p for p in live if p >= n_live)
    assert len(holes) == len(movers)
    new_page = {p: p for p in live}
    for hole, mover in zip(holes, movers):
        kv[:, :, hole] = kv[:, :, mover]
        new_page[mover] = hole
    bt_dst = np.full((n_keep, ppr), -1, dtype=np.int32)
    sl_dst = np.zeros(n_keep, dtype=np.int32)
    src_of_dst = np.full(n_keep, -1, dtype=np.int32)
    for r in range(n_keep):
        s = int(survivor_idx[r])
        if s < 0:
            continue
        for p, page in enumerate(pages_of[r]):
            bt_dst[r, p] = new_page[page]
        sl_dst[r] = seq_len_src[s]
        src_of_dst[r] = s
    return dict(block_table_dst=bt_dst, seq_len_dst=sl_dst, src_of_dst=src_of_dst,
                n_pages_used=n_live, n_moved=len(movers))


# ----------------------------------------------------------------------------
# 2-layer MLP quality head
# ----------------------------------------------------------------------------
def score_mlp(hidden_bits, w1_bits, b1, w2, b2=0.0):
    """Quality head as a 2-layer MLP (Sec. 4.2 allows a small two-layer MLP as the head) followed by the
    sigmoid normalisation of App. A.4.  Reading (the paper gives neither width nor activation):
        a = relu(W1 h + b1),  s = <w2, a> + b2,  q = sigmoid(s)
    hidden_bits [N, d] uint16 (bf16), w1_bits [m, d] uint16 (bf16), b1 [m] fp32, w2 [m] fp32.
    Returns (s, q) float64 [N]."""
    h = bf16_bits_to_f64(hidden_bits)
    W1 = bf16_bits_to_f64(w1_bits)
    b1 = np.asarray(b1, dtype=np.float32).astype(np.float64)
    w2 = np.asarray(w2, dtype=np.float32).astype(np.float64)
    n = h.shape[0]
    s = np.empty(n, dtype=np.float64)
    q = np.empty(n, dtype=np.float64)
    for i in range(n):
        pre = W1 @ h[i] + b1
        act = np.where(pre > 0.0, pre, 0.0)
        s[i] = math.fsum(act * w2) + float(b2)
        if s[i] >= 0.0:
            q[i] = 1.0 / (1.0 + math.exp(-s[i]))
        else:
            e = math.exp(s[i])
            q[i] = e / (1.0 + e)
    return s, q


# ----------------------------------------------------------------------------
# quality-head training: cross-entropy loss, its gradient, optimizer step
# ----------------------------------------------------------------------------
def _log_sigmoid(s):
    """log(sigmoid(s)) without overflow."""
    return -math.log1p(math.exp(-s)) if s >= 0.0 else s - math.log1p(math.exp(s))


def score_ce(hidden_bits, w, bias, labels):
    """Cross-entropy loss of the linear quality head against the final rewards (Sec. 4.2 and Sec. 4.3 (iii):
    the head is trained on the fly with a cross-entropy loss on the rollouts' rewards, the backbone's
    hidden state being a constant).  With q_i = sigmoid(<w, h_i> + bias) and label y_i in [0, 1]:
        L = -(1/N) sum_i [ y_i log q_i + (1 - y_i) log(1 - q_i) ]
    Returns L as a float (float64 arithmetic on the exact input values)."""
    h = bf16_bits_to_f64(hidden_bits)
    w = np.asarray(w, dtype=np.float32).astype(np.float64)
    y = np.asarray(labels, dtype=np.float32).astype(np.float64)
    n = h.shape[0]
    terms = []
    for i in range(n):
        s = math.fsum(h[i] * w) + float(bias)
        terms.append(-(y[i] * _log_sigmoid(s) + (1.0 - y[i]) * _log_sigmoid(-s)))
    return math.fsum(terms) / n


def score_ce_grad(hidden_bits, w, bias, labels):
    """Gradient of score_ce with respect to the head's parameters (the hidden states carry no gradient:
    Sec. 4.3 (iii) stops it at the backbone).  dL/ds_i = (q_i - y_i)/N, hence
        dL/dw = (1/N) sum_i (q_i - y_i) h_i,   dL/dbias = (1/N) sum_i (q_i - y_i).
    Returns (loss, grad_w float64 [d], grad_bias float)."""
    h = bf16_bits_to_f64(hidden_bits)
    wv = np.asarray(w, dtype=np.float32).astype(np.float64)
    y = np.asarray(labels, dtype=np.float32).astype(np.float64)
    n, d = h.shape
    r = np.empty(n, dtype=np.float64)
    for i in range(n):
        s = math.fsum(h[i] * wv) + float(bias)
        q = 1.0 / (1.0 + math.exp(-s)) if s >= 0.0 else math.exp(s) / (1.0 + math.exp(s))
        r[i] = q - y[i]
    grad_w = np.array([math.fsum(r * h[:, c]) for c in range(d)], dtype=np.float64) / n
    return score_ce(hidden_bits, w, bias, labels), grad_w, math.fsum(r) / n


def adamw_step(param, grad, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
    """One AdamW update (Alg. 1 updates the quality head in its optimizer step and names no optimizer;
    AdamW with decoupled weight decay, Loshchilov & Hutter 2019, is this build's reading):
        m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2
        p <- p - lr * ( (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps) + wd * p )
    `step` is t >= 1.  Inputs are taken at the precision they come in (fp32 from the library's buffers,
    float64 when a test carries the state over several steps); arithmetic in float64.
    Returns (param, m, v) float64."""
    p = np.asarray(param, dtype=np.float64)
    g = np.asarray(grad, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** step)
    v_hat = v / (1.0 - beta2 ** step)
    p = p - lr * (m_hat / (np.sqrt(v_hat) + eps) + weight_decay * p)
    return p, m, v


# ----------------------------------------------------------------------------
# trace confidence (Sec. 3, "Trace Confidence")
# ----------------------------------------------------------------------------
def token_confidence(hidden_bits, lm_head_bits):
    """Token confidence of Sec. 3: H_t = - sum_{j=1..V} log P_t(j), with P_t the softmax of the logits
    z_t = W h_t (temperature 1).  Written as the definition: every log-probability is formed, then summed.
    hidden_bits [T, d] uint16, lm_head_bits [V, d] uint16.  Returns float64 [T]."""
    T = hidden_bits.shape[0]
    W = bf16_bits_to_f64(lm_head_bits)
    out = np.empty(T, dtype=np.float64)
    for t in range(T):
        z = W @ bf16_bits_to_f64(hidden_bits[t])
        m = float(z.max())
        lse = m + math.log(math.fsum(np.exp(z - m)))
        out[t] = -math.fsum(z - lse)
    return out


def trace_confidence(conf, cu_seqlens, window, bottom_percent=10):
    """Trace-level aggregates of the token confidences (Sec. 3): for each trace i = tokens
    [cu[i], cu[i+1]):
      mean_i    the average token confidence over the trace (the self-uncertainty score),
      windows   H_w = mean of H_t over each run of `window` consecutive tokens (sliding by one token);
                a trace shorter than the window has the single window "the whole trace",
      min_i     the smallest window value,
      bottom_i  the average of the lowest ceil(bottom_percent/100 * n_windows) window values (at least
                one; integer arithmetic).
    An empty trace yields NaN.  conf float [T]; cu_seqlens int [n+1].  Returns three float64 [n] arrays."""
    conf = np.asarray(conf, dtype=np.float64)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    n = cu.shape[0] - 1
    mean = np.full(n, np.nan)
    wmin = np.full(n, np.nan)
    bottom = np.full(n, np.nan)
    for i in range(n):
        x = conf[cu[i]:cu[i + 1]]
        L = x.shape[0]
        if L == 0:
            continue
        mean[i] = math.fsum(x) / L
        w = min(int(window), L)
        vals = sorted(math.fsum(x[k:k + w]) / w for k in range(L - w + 1))
        wmin[i] = vals[0]
        m = max(1, (len(vals) * int(bottom_percent) + 99) // 100)
        bottom[i] = math.fsum(vals[:m]) / m
    return mean, wmin, bottom


# ----------------------------------------------------------------------------
# GRPO advantage and clipped-ratio objective (Sec. 3, "Group-Relative Policy Optimization")
# ----------------------------------------------------------------------------
def grpo_advantage(reward, group_offsets, ddof=0, eps=0.0):
    """Group-relative advantage of Sec. 3: A_i = (R_i - mean(R_group)) / std(R_group), over the rollouts of
    one prompt that are still there after pruning.  Rollouts of group g are [group_offsets[g],
    group_offsets[g+1]).  std = sqrt(sum (R - mean)^2 / (n - ddof)) (0 when n - ddof <= 0); `eps` is added to
    it; where std + eps == 0 (all rewards equal, the sparse-signal case the paper describes) A_i = 0.
    Returns float64 [N]."""
    r = np.asarray(reward, dtype=np.float32).astype(np.float64)
    off = np.asarray(group_offsets, dtype=np.int64)
    adv = np.zeros(r.shape[0], dtype=np.float64)
    for g in range(off.shape[0] - 1):
        x = r[off[g]:off[g + 1]]
        n = x.shape[0]
        if n == 0:
            continue
        mean = math.fsum(x) / n
        dev = x - mean
        std = math.sqrt(math.fsum(dev * dev) / (n - ddof)) if n - ddof > 0 else 0.0
        den = std + float(eps)
        adv[off[g]:off[g + 1]] = dev / den if den > 0.0 else 0.0
    return adv


def grpo_objective(logp, logp_ref, cu_seqlens, advantage, group_offsets, eps_low=0.2, eps_high=0.2, beta=0.0):
    """GRPO objective of Sec. 3 on the surviving rollouts:
        J = mean over groups g of (1/G_g) sum_{i in g} (1/|o_i|) sum_t [ min(r_t A_i, clip(r_t, 1-eps_low,
            1+eps_high) A_i) - beta * kl_t ],    r_t = exp(logp_t - logp_ref_t)
    with rollout i = tokens [cu[i], cu[i+1]).  The paper writes the KL term as beta * KL(pi_theta || pi_ref)
    without an estimator; the per-token estimate used is kl_t = exp(u) - u - 1 with u = logp_ref_t - logp_t
    (non-negative, and its expectation under pi_theta is the KL divergence).  An empty rollout adds 0.
    Returns (J, dJ/dlogp float64 [T], number of tokens where the clipped branch is strictly the minimum)."""
    lp = np.asarray(logp, dtype=np.float32).astype(np.float64)
    lr = np.asarray(logp_ref, dtype=np.float32).astype(np.float64)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    off = np.asarray(group_offsets, dtype=np.int64)
    adv = np.asarray(advantage, dtype=np.float32).astype(np.float64)
    n_groups = off.shape[0] - 1
    grad = np.zeros(lp.shape[0], dtype=np.float64)
    n_clipped = 0
    group_terms = []
    for g in range(n_groups):
        G = int(off[g + 1] - off[g])
        seq_terms = []
        for i in range(off[g], off[g + 1]):
            L = int(cu[i + 1] - cu[i])
            if L == 0:
                seq_terms.append(0.0)
                continue
            tok = []
            for t in range(cu[i], cu[i + 1]):
                ratio = math.exp(lp[t] - lr[t])
                plain = ratio * adv[i]
                clipped = min(max(ratio, 1.0 - eps_low), 1.0 + eps_high) * adv[i]
                u = lr[t] - lp[t]
                kl = math.exp(u) - u - 1.0
                tok.append(min(plain, clipped) - beta * kl)
                d = plain if plain <= clipped else 0.0            # d(min)/dlogp: r*A on the unclipped branch
                d -= beta * (1.0 - math.exp(u))                   # d(kl)/dlogp = 1 - exp(u)
                grad[t] = d / (L * G * n_groups)
                n_clipped += 1 if clipped < plain else 0
            seq_terms.append(math.fsum(tok) / L)
        group_terms.append(math.fsum(seq_terms) / G if G > 0 else 0.0)
    J = math.fsum(group_terms) / n_groups if n_groups > 0 else 0.0
    return J, grad, n_clipped


# ----------------------------------------------------------------------------
# training the 2-layer MLP head
# ----------------------------------------------------------------------------
def score_mlp_ce_grad(hidden_bits, w1_bits, b1, w2, b2, labels):
    """Cross-entropy loss of the MLP head of score_mlp (a = relu(W1 h + b1), s = <w2, a> + b2,
    q = sigmoid(s)) against the rewards, mean over the rows, and its gradient with respect to every head
    parameter; the hidden states are constants (Sec. 4.2, Sec. 4.3 (iii)).  With r_i = (q_i - y_i)/N:
        dL/db2 = sum_i r_i                 dL/dw2 = sum_i r_i a_i
        delta_i = r_i * w2 * [W1 h_i + b1 > 0]
        dL/db1 = sum_i delta_i             dL/dW1 = sum_i delta_i h_i^T
    (ReLU's derivative at 0 is taken as 0.)  Returns (loss, gW1 [m, d], gb1 [m], gw2 [m], gb2), float64."""
    h = bf16_bits_to_f64(hidden_bits)
    W1 = bf16_bits_to_f64(w1_bits)
    b1 = np.asarray(b1, dtype=np.float32).astype(np.float64)
    w2 = np.asarray(w2, dtype=np.float32).astype(np.float64)
    y = np.asarray(labels, dtype=np.float32).astype(np.float64)
    n = h.shape[0]
    m = W1.shape[0]
    gW1 = np.zeros_like(W1)
    gb1 = np.zeros(m)
    gw2 = np.zeros(m)
    gb2 = 0.0
    terms = []
    for i in range(n):
        pre = W1 @ h[i] + b1
        act = np.where(pre > 0.0, pre, 0.0)
        s = math.fsum(act * w2) + float(b2)
        terms.append(-(y[i] * _log_sigmoid(s) + (1.0 - y[i]) * _log_sigmoid(-s)))
        q = 1.0 / (1.0 + math.exp(-s)) if s >= 0.0 else math.exp(s) / (1.0 + math.exp(s))
        r = (q - y[i]) / n
        delta = np.where(pre > 0.0, r * w2, 0.0)
        gb2 += r
        gw2 += r * act
        gb1 += delta
        gW1 += np.outer(delta, h[i])
    return math.fsum(terms) / n, gW1, gb1, gw2, gb2
