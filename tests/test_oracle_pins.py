"""Pins for the CPU oracle: every oracle function is checked against something
other than itself -- closed forms, invariants, exact-rational brute force of the
paper's definitions, and hand-derived examples.  The paper prints no worked
numeric example for any stage, so there are no paper-printed goldens."""
import itertools
import math
import random
from fractions import Fraction

import numpy as np
import pytest

import oracle as O


def f32_to_bf16_bits(x):
    """Round-to-nearest-even float32 -> bf16 bit patterns (test-side helper)."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def bits_to_fraction(b):
    """Exact rational value of one bf16 bit pattern (finite)."""
    b = int(b)
    sign = -1 if b >> 15 else 1
    e = (b >> 7) & 0xFF
    m = b & 0x7F
    if e == 0:
        return sign * Fraction(m, 1 << 7) * Fraction(1, 1 << 126)
    return sign * (1 + Fraction(m, 1 << 7)) * (Fraction(2) ** (e - 127))


# ----------------------------------------------------------------------------- bf16
def test_bf16_widening_is_exact():
    vals = np.array([0.0, 1.0, -2.0, 0.5, 1.5, 3.140625, -0.0078125], dtype=np.float32)
    bits = f32_to_bf16_bits(vals)
    out = O.bf16_bits_to_f64(bits)
    assert np.array_equal(out, vals.astype(np.float64))
    for b, v in zip(bits, out):
        assert bits_to_fraction(b) == Fraction(float(v))


# ----------------------------------------------------------------------------- score
def test_score_zero_weight_gives_half():
    rng = np.random.default_rng(1)
    h = f32_to_bf16_bits(rng.standard_normal((5, 16)))
    s, q = O.score(h, np.zeros(16, np.float32), 0.0)
    assert np.all(s == 0.0) and np.all(q == 0.5)


def test_score_one_hot_picks_weight():
    d = 24
    rng = np.random.default_rng(2)
    w = rng.standard_normal(d).astype(np.float32)
    for k, c in [(0, 1.5), (7, -2.0), (23, 0.25)]:
        h = np.zeros((1, d), np.float32)
        h[0, k] = c
        s, q = O.score(f32_to_bf16_bits(h), w, 0.0)
        assert s[0] == c * float(w[k])
        assert abs(q[0] - 0.5 * (1.0 + math.tanh(0.5 * s[0]))) < 1e-15


def test_score_exact_rational_dot_and_bias():
    rng = np.random.default_rng(3)
    N, d = 4, 32
    hb = f32_to_bf16_bits(rng.standard_normal((N, d)))
    w = rng.standard_normal(d).astype(np.float32)
    bias = 0.375
    s, q = O.score(hb, w, bias)
    for i in range(N):
        exact = sum(bits_to_fraction(hb[i, k]) * Fraction(float(w[k])) for k in range(d)) + Fraction(bias)
        assert abs(s[i] - float(exact)) <= 1e-14 * max(1.0, abs(float(exact)))
        # sigmoid through the tanh identity, an independent closed form
        assert abs(q[i] - 0.5 * (1.0 + math.tanh(0.5 * float(exact)))) < 1e-14


def test_score_symmetry_monotone_saturation():
    rng = np.random.default_rng(4)
    h = rng.standard_normal((16, 8)).astype(np.float32)
    hb = f32_to_bf16_bits(h)
    hb_neg = hb ^ np.uint16(0x8000)            # exact negation of every element
    w = rng.standard_normal(8).astype(np.float32)
    s, q = O.score(hb, w)
    s2, q2 = O.score(hb_neg, w)
    assert np.allclose(s2, -s, rtol=0, atol=0)
    assert np.allclose(q + q2, 1.0, rtol=0, atol=1e-15)
    order = np.argsort(s)
    assert np.all(np.diff(q[order]) >= 0)
    for b, lo, hi in [(100.0, 1.0 - 1e-40, 1.0), (-100.0, 0.0, 1e-40)]:
        _, qq = O.score(hb[:1], np.zeros(8, np.float32), b)
        assert np.isfinite(qq[0]) and lo <= qq[0] <= hi
    _, qq = O.score(hb[:1], np.zeros(8, np.float32), -1000.0)
    assert qq[0] == 0.0


# ----------------------------------------------------------------------------- select
def definition_in_rationals(q_frac, K, rho):
    """The paper's rule evaluated literally in exact rationals (Thm 4.2):
    mu_{-j} = mean of the live probabilities without j; prune argmin |mu_{-j}-rho|,
    first index on ties; repeat until K remain."""
    live = list(range(len(q_frac)))
    order = []
    while len(live) > K:
        devs = []
        for j in live:
            others = [q_frac[i] for i in live if i != j]
            mu = sum(others) / len(others)
            devs.append(abs(mu - rho))
        j_hat = live[devs.index(min(devs))]
        live.remove(j_hat)
        order.append(j_hat)
    return live, order


def test_select_matches_rational_definition_random():
    rnd = random.Random(7)
    for trial in range(300):
        G = rnd.randint(2, 9)
        K = rnd.randint(1, G)
        if trial % 3 == 0:   # coarse grid: many exact ties
            q = np.array([rnd.randint(0, 16) / 16.0 for _ in range(G)], dtype=np.float32)
        else:
            q = np.array([rnd.random() for _ in range(G)], dtype=np.float32)
        rho32 = np.float32(rnd.choice([0.5, 0.25, 0.7, 0.0, 1.0]))
        k = O.quantise(q)
        R = O.quantise(np.array([rho32]))[0]
        q_frac = [Fraction(v, 1 << 30) for v in k]
        live_def, order_def = definition_in_rationals(q_frac, K, Fraction(R, 1 << 30))
        live, order = O.select_group(k, K, R)
        assert live == live_def and order == order_def
        # the batched entry point with this rho: two copies of the group, second one reversed
        keep, surv = O.select(np.concatenate([q, q[::-1]]), 2, G, K, float(rho32))
        assert [int(i) for i in surv[:K]] == live_def
        live_rev, _ = definition_in_rationals(q_frac[::-1], K, Fraction(R, 1 << 30))
        assert [int(i) - G for i in surv[K:]] == live_rev
        assert keep.sum() == 2 * K and all(keep[i] for i in surv)


def test_select_closed_form_closest_to_t():
    # |mu_{-j} - rho| = |S - q_j - rho (n-1)| / (n-1): the pruned rollout is the
    # live one closest to t = S - rho (n-1)
    rnd = random.Random(11)
    for _ in range(200):
        G = rnd.randint(2, 16)
        k = [rnd.randint(0, 1 << 30) for _ in range(G)]
        R = rnd.randint(0, 1 << 30)
        live, order = O.select_group(k, G - 1, R)
        t = sum(k) - R * (G - 1)
        dist = [abs(v - t) for v in k]
        assert order[0] == dist.index(min(dist))


def test_select_quantise_is_round_half_even_on_fp32():
    q = np.array([0.5, 0.25, 1.0, 0.0, 2.0 ** -31, 3 * 2.0 ** -31, 1 - 2.0 ** -24], dtype=np.float32)
    assert O.quantise(q) == [1 << 29, 1 << 28, 1 << 30, 0, 0, 2, (1 << 30) - 64]


def test_select_hand_worked_examples():
    # derived by hand from the rule with rho = 0.5, using t = S - rho (n-1):
    # q=[.9,.6,.3,.1]: t=.4 -> drop .3 (idx 2); t=1.6-1.0=.6 -> drop idx 1.
    k = O.quantise(np.array([0.9, 0.6, 0.3, 0.1], np.float32))
    assert O.select_group(k, 2, 1 << 29) == ([0, 3], [2, 1])
    # q=[.95,.9,.8,.7,.65,.3,.2,.05]: S=4.55,t=1.05 -> idx0; S=3.6,t=.6 -> idx4 (.65);
    # S=2.95,t=.45 -> idx5 (.3, dist .15 < .25); S=2.65,t=.65 -> idx3 (.7)
    k = O.quantise(np.array([0.95, 0.9, 0.8, 0.7, 0.65, 0.3, 0.2, 0.05], np.float32))
    assert O.select_group(k, 4, 1 << 29) == ([1, 2, 6, 7], [0, 4, 5, 3])
    # low-probability group: t is below every q for a while, so minima go first
    k = O.quantise(np.array([0.1, 0.1, 0.2, 0.05, 0.3, 0.15, 0.1, 0.9], np.float32))
    assert O.select_group(k, 4, 1 << 29) == ([2, 4, 5, 7], [3, 0, 1, 6])
    # all equal: every step is an exact tie -> lowest index goes
    k = O.quantise(np.full(8, 0.5, np.float32))
    assert O.select_group(k, 4, 1 << 29) == ([4, 5, 6, 7], [0, 1, 2, 3])


def test_select_lemma_4_1_strict_improvement():
    # Lemma 4.1: if mu > rho and some q_j > mu (or the mirror case), pruning that j
    # moves the mean toward rho, by mu_{-j} - mu = (mu - q_j)/(G-1).  The lemma's
    # proof does not consider a step that jumps past rho (possible for small G), so
    # the strict decrease is asserted only when that j does not overshoot; the
    # argmin rule is at least as good as that j.
    rnd = random.Random(5)
    hits = 0
    for _ in range(2000):
        G = rnd.randint(3, 12)
        k = [rnd.randint(0, 1 << 30) for _ in range(G)]
        R = rnd.randint(0, 1 << 30)
        mu = Fraction(sum(k), G)
        good = []
        for j in range(G):
            mu_j = Fraction(sum(k) - k[j], G - 1)
            assert mu_j - mu == (mu - k[j]) / (G - 1)
            if (mu > R and k[j] > mu and mu_j >= R) or (mu < R and k[j] < mu and mu_j <= R):
                good.append(j)
        if not good:
            continue
        hits += 1
        live, _ = O.select_group(k, G - 1, R)
        mu_after = Fraction(sum(k[i] for i in live), G - 1)
        assert abs(mu_after - R) < abs(mu - R)
    assert hits > 300


def test_select_outputs_exactly_k_sorted_and_group_independent():
    rng = np.random.default_rng(9)
    n_groups, G, K = 6, 8, 3
    p = rng.random(n_groups * G).astype(np.float32)
    keep, surv = O.select(p, n_groups, G, K, 0.5)
    assert keep.dtype == np.uint8 and surv.dtype == np.int32
    assert keep.reshape(n_groups, G).sum(axis=1).tolist() == [K] * n_groups
    assert np.array_equal(np.flatnonzero(keep), surv)
    # groups are independent: permuting whole groups permutes the result
    perm = rng.permutation(n_groups)
    p2 = p.reshape(n_groups, G)[perm].reshape(-1)
    keep2, _ = O.select(p2, n_groups, G, K, 0.5)
    assert np.array_equal(keep2.reshape(n_groups, G), keep.reshape(n_groups, G)[perm])
    # K == G keeps everything; bad K is rejected
    keep3, surv3 = O.select(p, n_groups, G, G, 0.5)
    assert keep3.all() and np.array_equal(surv3, np.arange(n_groups * G))
    with pytest.raises(ValueError):
        O.select(p, n_groups, G, 0, 0.5)
    with pytest.raises(ValueError):
        O.select(p, n_groups, G, G + 1, 0.5)


def test_select_not_worse_than_random_subset_on_average():
    # sanity, not parity: the greedy rule's |mean - rho| is far below a random K-subset's
    rng = np.random.default_rng(13)
    G, K = 16, 8
    dev_sel, dev_rnd = 0.0, 0.0
    for _ in range(200):
        p = rng.beta(0.5, 0.5, G).astype(np.float32)
        _, surv = O.select(p, 1, G, K, 0.5)
        dev_sel += abs(float(p[surv].mean()) - 0.5)
        dev_rnd += abs(float(p[rng.permutation(G)[:K]].mean()) - 0.5)
    assert dev_sel < 0.5 * dev_rnd


# ----------------------------------------------------------------------------- compact
def make_paged(rng, N, ppr, page_tokens, L=2, H=2, hd=4, seq_lens=None, extra_pages=3, max_len=None):
    P = N * ppr + extra_pages
    kv = rng.integers(0, 1 << 16, size=(L, 2, P, page_tokens, H, hd), dtype=np.uint16)
    bt = rng.permutation(P)[:N * ppr].reshape(N, ppr).astype(np.int32)
    if seq_lens is None:
        seq_lens = np.full(N, ppr * page_tokens, np.int32)
    max_len = max_len or ppr * page_tokens
    tokens = rng.integers(0, 1000, size=(N, max_len), dtype=np.int32)
    return kv, bt, np.asarray(seq_lens, np.int32), tokens


def test_compact_logical_content_is_preserved():
    rng = np.random.default_rng(21)
    N, ppr, pt = 7, 4, 4
    seq = rng.integers(1, ppr * pt + 1, size=N).astype(np.int32)
    kv, bt, seq, tok = make_paged(rng, N, ppr, pt, seq_lens=seq)
    surv = np.array([1, 2, 5, 6], np.int32)
    out = O.compact(kv, bt, seq, tok, surv, n_pages_dst=len(surv) * ppr)
    used = 0
    for r, src in enumerate(surv):
        assert out["seq_len_dst"][r] == seq[src] and out["src_of_dst"][r] == src
        assert np.array_equal(out["tokens_dst"][r], tok[src])
        n_pages = -(-int(seq[src]) // pt)
        assert out["block_table_dst"][r, :n_pages].tolist() == list(range(used, used + n_pages))
        assert np.all(out["block_table_dst"][r, n_pages:] == -1)
        for t in range(int(seq[src])):          # read token t through either table
            p, o = divmod(t, pt)
            a = kv[:, :, bt[src, p], o]
            b = out["kv_dst"][:, :, out["block_table_dst"][r, p], o]
            assert np.array_equal(a, b)
        used += n_pages
    assert out["n_pages_used"] == used
    # destination pages past n_pages_used are untouched
    assert np.all(out["kv_dst"][:, :, used:] == 0)


def test_compact_equals_library_gather_and_ignores_pruned_pages():
    rng = np.random.default_rng(22)
    N, ppr, pt = 8, 3, 2
    kv, bt, seq, tok = make_paged(rng, N, ppr, pt)
    surv = np.array([0, 3, 4, 7], np.int32)
    out = O.compact(kv, bt, seq, tok, surv, n_pages_dst=len(surv) * ppr)
    flat_src_pages = bt[surv].reshape(-1)
    assert np.array_equal(out["kv_dst"], np.take(kv, flat_src_pages, axis=2))
    # poison every page that belongs to no survivor: result must not change
    kv2 = kv.copy()
    dead = np.setdiff1d(np.arange(kv.shape[2]), flat_src_pages)
    kv2[:, :, dead] = 0x7FC0  # bf16 NaN pattern
    out2 = O.compact(kv2, bt, seq, tok, surv, n_pages_dst=len(surv) * ppr)
    assert np.array_equal(out2["kv_dst"], out["kv_dst"])
    assert not np.any(out2["kv_dst"] == 0x7FC0) or np.any(kv[:, :, flat_src_pages] == 0x7FC0)


def test_compact_identity_and_page_permutation_invariance():
    rng = np.random.default_rng(23)
    N, ppr, pt = 4, 2, 4
    kv, bt, seq, tok = make_paged(rng, N, ppr, pt, extra_pages=0)
    dense = np.arange(N * ppr, dtype=np.int32).reshape(N, ppr)
    out = O.compact(kv, dense, seq, tok, np.arange(N, dtype=np.int32), n_pages_dst=N * ppr)
    assert np.array_equal(out["kv_dst"], kv) and np.array_equal(out["block_table_dst"], dense)
    # relabel physical pages: move page p to sigma[p], rewrite the table -> same result
    surv = np.array([1, 3], np.int32)
    ref = O.compact(kv, bt, seq, tok, surv, n_pages_dst=4)
    sigma = rng.permutation(kv.shape[2])
    kv_perm = np.empty_like(kv)
    kv_perm[:, :, sigma] = kv
    out_perm = O.compact(kv_perm, sigma[bt].astype(np.int32), seq, tok, surv, n_pages_dst=4)
    assert np.array_equal(out_perm["kv_dst"], ref["kv_dst"])


# ----------------------------------------------------------------------------- logprob
def test_logprob_full_distribution_sums_to_one():
    rng = np.random.default_rng(31)
    h = f32_to_bf16_bits(rng.standard_normal((6, 16)))
    W = f32_to_bf16_bits(rng.standard_normal((50, 16)))
    full, lse = O.log_softmax_rows(h, W)
    assert np.all(np.abs(np.exp(full).sum(axis=1) - 1.0) < 1e-12)
    tg = rng.integers(0, 50, 6)
    lp, lse2 = O.logprob(h, W, tg)
    assert np.allclose(lp, full[np.arange(6), tg], rtol=0, atol=1e-13)
    assert np.allclose(lse, lse2, rtol=0, atol=1e-13)


def test_logprob_zero_head_is_uniform_and_single_class():
    rng = np.random.default_rng(32)
    h = f32_to_bf16_bits(rng.standard_normal((3, 8)))
    V = 37
    lp, lse = O.logprob(h, np.zeros((V, 8), np.uint16), np.array([0, 5, 36]))
    assert np.allclose(lp, -math.log(V), rtol=0, atol=1e-15)
    assert np.allclose(lse, math.log(V), rtol=0, atol=1e-15)
    lp1, _ = O.logprob(h, f32_to_bf16_bits(rng.standard_normal((1, 8))), np.zeros(3, int))
    assert np.all(lp1 == 0.0)


def test_logprob_two_class_closed_form():
    # V = 2: log p(target) = -log(1 + exp(z_other - z_target)) with exact rational logits
    rng = np.random.default_rng(33)
    d = 12
    hb = f32_to_bf16_bits(rng.standard_normal((5, d)))
    Wb = f32_to_bf16_bits(rng.standard_normal((2, d)))
    tg = np.array([0, 1, 1, 0, 1])
    lp, _ = O.logprob(hb, Wb, tg)
    for t in range(5):
        z = [float(sum(bits_to_fraction(hb[t, k]) * bits_to_fraction(Wb[v, k]) for k in range(d)))
             for v in range(2)]
        expect = -math.log1p(math.exp(z[1 - tg[t]] - z[tg[t]]))
        assert abs(lp[t] - expect) < 1e-13


def test_logprob_pure_python_brute_force():
    rng = np.random.default_rng(34)
    T, V, d = 3, 7, 5
    hb = f32_to_bf16_bits(rng.standard_normal((T, d)))
    Wb = f32_to_bf16_bits(rng.standard_normal((V, d)))
    tg = [6, 0, 3]
    lp, lse = O.logprob(hb, Wb, tg)
    for t in range(T):
        z = [float(sum(bits_to_fraction(hb[t, k]) * bits_to_fraction(Wb[v, k]) for k in range(d)))
             for v in range(V)]
        denom = math.fsum(math.exp(x) for x in z)
        assert abs(lp[t] - (z[tg[t]] - math.log(denom))) < 1e-13
        assert abs(lse[t] - math.log(denom)) < 1e-13


def test_logprob_shift_invariance_and_dominant_logit():
    rng = np.random.default_rng(35)
    T, V, d = 4, 20, 8
    h = rng.standard_normal((T, d)).astype(np.float32)
    W = rng.standard_normal((V, d)).astype(np.float32)
    tg = rng.integers(0, V, T)
    lp, lse = O.logprob(f32_to_bf16_bits(h), f32_to_bf16_bits(W), tg)
    # an extra feature h=1 with the same weight c on every vocab row adds c to every logit
    h2 = np.concatenate([h, np.ones((T, 1), np.float32)], axis=1)
    W2 = np.concatenate([W, np.full((V, 1), 3.5, np.float32)], axis=1)
    lp2, lse2 = O.logprob(f32_to_bf16_bits(h2), f32_to_bf16_bits(W2), tg)
    assert np.allclose(lp2, lp, rtol=0, atol=1e-12)
    assert np.allclose(lse2, lse + 3.5, rtol=0, atol=1e-12)
    # one dominant logit on the target -> log-prob -> 0; on another row -> about -gap
    hd = np.zeros((1, d), np.float32); hd[0, 0] = 64.0
    Wd = np.zeros((V, d), np.float32); Wd[4, 0] = 1.0
    lpd, _ = O.logprob(f32_to_bf16_bits(hd), f32_to_bf16_bits(Wd), [4])
    assert -1e-20 > lpd[0] > -1e-10 or lpd[0] == 0.0 or abs(lpd[0]) < 1e-10
    lpo, _ = O.logprob(f32_to_bf16_bits(hd), f32_to_bf16_bits(Wd), [5])
    assert abs(lpo[0] + 64.0) < 1e-9


# ----------------------------------------------------------------------------- vote
def test_vote_worked_example_and_rank_sum():
    # q=[.2,.9,.9,.4]: ranks 0, (2+3)/2, (2+3)/2, 1 -> doubled [0,5,5,2]
    w, tally = O.weighted_vote(np.array([0.2, 0.9, 0.9, 0.4], np.float32), [1, 0, 2, 1], 1, 4, 3)
    assert tally.tolist() == [[5, 2, 5]] and w.tolist() == [0]   # majority vote would say 1
    rng = np.random.default_rng(41)
    for C in [1, 2, 5, 16]:
        q = rng.integers(0, 6, C).astype(np.float32) / 8  # ties likely
        ans = rng.integers(0, 4, C)
        _, t = O.weighted_vote(q, ans, 1, C, 4)
        assert t.sum() == C * (C - 1)


def test_vote_distinct_scores_give_linear_ranks():
    # no ties: sorted position r has weight r/(C-1) in [0,1]  (rank2 = 2r)
    q = np.array([0.3, 0.1, 0.8, 0.5, 0.9], np.float32)
    _, t = O.weighted_vote(q, [0, 1, 2, 3, 4], 1, 5, 5)
    assert t[0].tolist() == [2, 0, 6, 4, 8]
    weights = t[0] / (2.0 * (5 - 1))
    assert weights.min() == 0.0 and weights.max() == 1.0


def test_vote_equal_scores_reduce_to_majority():
    rng = np.random.default_rng(42)
    for _ in range(50):
        C, A = 9, 4
        ans = rng.integers(0, A, C)
        w, _ = O.weighted_vote(np.full(C, 0.3, np.float32), ans, 1, C, A)
        counts = np.bincount(ans, minlength=A)
        assert w[0] == int(np.argmax(counts))       # first max = lowest id on ties


def test_vote_invariances_and_single_candidate():
    rng = np.random.default_rng(43)
    Q, C, A = 5, 12, 6
    q = rng.random(Q * C).astype(np.float32)
    ans = rng.integers(0, A, Q * C)
    w, t = O.weighted_vote(q, ans, Q, C, A)
    perm = rng.permutation(C)
    qp = q.reshape(Q, C)[:, perm].reshape(-1)
    ap = ans.reshape(Q, C)[:, perm].reshape(-1)
    w2, t2 = O.weighted_vote(qp, ap, Q, C, A)
    assert np.array_equal(w, w2) and np.array_equal(t, t2)
    w3, t3 = O.weighted_vote((q * 4 - 2).astype(np.float32) ** 3, ans, Q, C, A)  # increasing map
    assert np.array_equal(w, w3) and np.array_equal(t, t3)
    w1, t1 = O.weighted_vote(np.array([0.7], np.float32), [3], 1, 1, 5)
    assert w1.tolist() == [3] and t1.sum() == 0      # absent ids never win


# ----------------------------------------------------------------------------- practical policy (App. A.4)
def test_bin_index_edges_and_histogram_brute_force():
    B = 128
    s = np.array([0.0, 1.0, 0.5, 127 / 128, 1 / 128, np.nextafter(np.float32(1 / 128), np.float32(0)), 0.999999],
                 dtype=np.float32)
    assert O.bin_index(s, B).tolist() == [0, 127, 64, 127, 1, 0, 127]
    rng = np.random.default_rng(51)
    s = rng.random(500).astype(np.float32)
    lab = rng.integers(0, 2, 500)
    for B in (128, 10, 1):
        c_pos, c_neg = O.histogram(s, lab, B)
        assert c_pos.sum() == lab.sum() and c_neg.sum() == 500 - lab.sum()
        for b in range(B):  # definition with exact rationals: b <= B s' < b+1 (the top edge closed for the last bin)
            inside = [(Fraction(float(np.float32(x) * np.float32(B))) >= b) and
                      (Fraction(float(np.float32(x) * np.float32(B))) < b + 1 or b == B - 1) for x in s]
            assert c_pos[b] == sum(1 for k in range(500) if inside[k] and lab[k])
            assert c_neg[b] == sum(1 for k in range(500) if inside[k] and not lab[k])


def test_posterior_alpha_zero_is_the_empirical_fraction():
    # with alpha = 0 Bayes' rule collapses: pi P(b|1) = c_b^+ / N, so q(b) = c_b^+ / (c_b^+ + c_b^-)
    rng = np.random.default_rng(52)
    c_pos = rng.integers(1, 50, 16)
    c_neg = rng.integers(1, 50, 16)
    q, pi = O.posterior_lut(c_pos, c_neg, 0.0)
    assert np.allclose(q, c_pos / (c_pos + c_neg), rtol=0, atol=1e-15)
    assert abs(pi - c_pos.sum() / (c_pos.sum() + c_neg.sum())) < 1e-15


def test_posterior_uninformative_histograms_return_the_prior():
    # identical class-conditional histograms carry no information: q(b) = pi in every bin
    c = np.array([3, 0, 7, 1, 9, 2])
    q, pi = O.posterior_lut(2 * c, c, 0.0 + 1e-300)
    assert np.allclose(q[c > 0], 2 / 3, rtol=0, atol=1e-12) and abs(pi - 2 / 3) < 1e-15
    # heavy smoothing washes the likelihoods out: q -> pi
    rng = np.random.default_rng(53)
    c_pos, c_neg = rng.integers(0, 30, 8), rng.integers(0, 30, 8)
    q, pi = O.posterior_lut(c_pos, c_neg, 1e12)
    assert np.allclose(q, pi, rtol=0, atol=1e-9)
    # empty buffers: prior 1/2 everywhere
    q, pi = O.posterior_lut(np.zeros(4), np.zeros(4), 1.0)
    assert pi == 0.5 and np.all(q == 0.5)
    # likelihoods are distributions over bins
    for a in (0.5, 1.0, 3.0):
        lp = (c_pos + a) / (c_pos.sum() + a * 8)
        assert abs(lp.sum() - 1.0) < 1e-15


def test_posterior_exact_rational_bayes():
    c_pos, c_neg, alpha = [5, 0, 2], [1, 4, 0], Fraction(1, 2)
    q, _ = O.posterior_lut(c_pos, c_neg, float(alpha))
    B, n_pos, n_neg = 3, sum(c_pos), sum(c_neg)
    pi = Fraction(n_pos, n_pos + n_neg)
    for b in range(B):
        l1 = (c_pos[b] + alpha) / (n_pos + alpha * B)
        l0 = (c_neg[b] + alpha) / (n_neg + alpha * B)
        assert abs(q[b] - float(pi * l1 / (pi * l1 + (1 - pi) * l0))) < 1e-15


def test_survival_closed_form_without_clipping():
    # if no bin is clipped, E[kappa + delta + lambda (rho - q)] = kappa gives delta = lambda (E[q] - rho)
    rng = np.random.default_rng(54)
    q = rng.uniform(0.3, 0.7, 32)
    w = rng.random(32); w /= w.sum()
    p, delta = O.survival_lut(q, w, kappa=0.5, rho=0.5, lam=0.5, p_min=0.0, p_max=1.0)
    assert abs(delta - 0.5 * (float(np.dot(w, q)) - 0.5)) < 1e-12
    assert np.allclose(p, 0.5 + delta + 0.5 * (0.5 - q), rtol=0, atol=1e-12)
    assert abs(float(np.dot(w, p)) - 0.5) < 1e-12
    # lambda = 0: every rollout survives with probability kappa, delta = 0
    p, delta = O.survival_lut(q, w, 0.25, 0.5, 0.0, 0.05, 0.95)
    assert abs(delta) < 1e-12 and np.allclose(p, 0.25, rtol=0, atol=1e-12)


def test_survival_with_clipping_keeps_the_rate_and_the_order():
    rng = np.random.default_rng(55)
    for _ in range(50):
        B = 128
        q = rng.beta(0.4, 0.4, B)
        w = rng.random(B) ** 3; w /= w.sum()
        kappa, rho, lam = rng.choice([0.25, 0.5, 0.75]), rng.choice([0.3, 0.5]), rng.choice([0.5, 1.0, 2.0])
        p_min, p_max = 0.05, 0.95
        p, delta = O.survival_lut(q, w, kappa, rho, lam, p_min, p_max)
        assert np.all(p >= p_min) and np.all(p <= p_max)
        assert abs(float(np.dot(w, p)) - kappa) < 1e-9                  # expected keep rate = kappa
        order = np.argsort(q)
        assert np.all(np.diff(p[order]) <= 1e-15)                       # monotone: likelier-correct rollouts are kept less
        # brute force: delta is a root of the (monotone) keep-rate curve
        f = lambda d: float(np.dot(w, np.clip(kappa + d + lam * (rho - q), p_min, p_max))) - kappa
        assert f(delta - 1e-6) <= 1e-9 and f(delta + 1e-6) >= -1e-9
    # unattainable target: kappa below p_min -> everything clipped at p_min
    p, _ = O.survival_lut(q, w, 0.01, 0.5, 0.5, 0.05, 0.95)
    assert np.allclose(p, 0.05, rtol=0, atol=1e-9)


def test_calibrate_composes_and_tilts_toward_low_posteriors():
    # rollouts with a high posterior get a lower survival probability than those with a low one
    c_pos = np.array([1, 2, 4, 8, 16, 32, 64, 128])
    c_neg = c_pos[::-1].copy()
    q, p, delta = O.calibrate(c_pos, c_neg, 0.5, 0.5, 0.5, 0.05, 0.95, 1.0)
    assert np.all(np.diff(q) > 0) and np.all(np.diff(p) < 0)
    w = O.bin_weights(c_pos, c_neg)
    assert abs(float(np.dot(w, p)) - 0.5) < 1e-9
    # p falls as q rises, so the kept set can only hold a lower share of likely-correct rollouts than the
    # population (Chebyshev's sum inequality); nothing in Eq. 2 stops it from overshooting rho
    kept_pos_rate = float(np.dot(w * p, q) / np.dot(w, p))
    assert kept_pos_rate <= float(np.dot(w, q)) + 1e-12


def test_prune_bernoulli_decisions_and_rate():
    rng = np.random.default_rng(56)
    B = 128
    p_lut = np.linspace(0.9, 0.1, B).astype(np.float32)
    s = rng.random(2000).astype(np.float32)
    u = rng.random(2000).astype(np.float32)
    p, keep, surv, n = O.prune_bernoulli(s, u, p_lut)
    assert np.array_equal(p, p_lut[np.minimum(B - 1, np.floor(s * 128).astype(int))])
    assert n == int(keep.sum()) == len(surv) and np.array_equal(surv, np.flatnonzero(u < p))
    assert abs(n / 2000 - 0.5) < 0.05                                  # E[p] = 0.5 under uniform scores
    _, keep0, _, n0 = O.prune_bernoulli(s, np.zeros(2000, np.float32), p_lut)
    _, keep1, _, n1 = O.prune_bernoulli(s, np.ones(2000, np.float32), p_lut)
    assert n0 == 2000 and n1 == 0


# ----------------------------------------------------------------------------- in-place compaction
def test_compact_inplace_dense_prefix_content_and_minimal_moves():
    rng = np.random.default_rng(61)
    for trial in range(20):
        N, ppr, pt = 9, 4, 4
        seq = rng.integers(1, ppr * pt + 1, size=N).astype(np.int32)
        kv, bt, seq, tok = make_paged(rng, N, ppr, pt, seq_lens=seq, extra_pages=int(rng.integers(0, 6)))
        surv = np.sort(rng.choice(N, size=int(rng.integers(1, N + 1)), replace=False)).astype(np.int32)
        before = kv.copy()
        out = O.compact_inplace(kv, bt, seq, surv)
        n_live = out["n_pages_used"]
        used = []
        for r, s in enumerate(surv):
            n_pages = -(-int(seq[s]) // pt)
            row = out["block_table_dst"][r]
            assert np.all(row[n_pages:] == -1) and np.all(row[:n_pages] >= 0) and np.all(row[:n_pages] < n_live)
            used.extend(row[:n_pages].tolist())
            for t in range(int(seq[s])):                     # every token reads the same bytes as before
                p, o = divmod(t, pt)
                assert np.array_equal(kv[:, :, row[p], o], before[:, :, bt[s, p], o])
            assert out["seq_len_dst"][r] == seq[s] and out["src_of_dst"][r] == s
        assert sorted(used) == list(range(n_live))           # the prefix is dense and nothing is shared
        # minimality: a page must move iff it is live and lies outside the prefix; everything else is untouched
        live_before = set(int(bt[s, p]) for s in surv for p in range(-(-int(seq[s]) // pt)))
        must_move = [p for p in live_before if p >= n_live]
        assert out["n_moved"] == len(must_move)
        changed = [p for p in range(kv.shape[2]) if not np.array_equal(kv[:, :, p], before[:, :, p])]
        assert len(changed) <= out["n_moved"] and all(p < n_live and p not in live_before for p in changed)


def test_compact_inplace_identity_and_pairing_order():
    rng = np.random.default_rng(62)
    N, ppr, pt = 4, 2, 2
    kv, _, seq, _ = make_paged(rng, N, ppr, pt, extra_pages=0)
    dense = np.arange(N * ppr, dtype=np.int32).reshape(N, ppr)
    before = kv.copy()
    out = O.compact_inplace(kv, dense, seq, np.array([0, 1], np.int32))     # survivors already form the prefix
    assert out["n_moved"] == 0 and np.array_equal(kv, before) and np.array_equal(out["block_table_dst"], dense[:2])
    # survivors 2,3 own pages 4..7: holes 0..3 are filled in ascending order by movers 4..7
    out = O.compact_inplace(kv, dense, seq, np.array([2, 3], np.int32))
    assert out["n_moved"] == 4 and out["block_table_dst"].tolist() == [[0, 1], [2, 3]]
    assert np.array_equal(kv[:, :, 0:4], before[:, :, 4:8])
    # an empty survivor set frees everything
    out = O.compact_inplace(kv, dense, seq, np.array([], np.int32))
    assert out["n_pages_used"] == 0 and out["n_moved"] == 0


# ----------------------------------------------------------------------------- MLP head
def test_score_mlp_reduces_to_the_linear_head_when_relu_is_inactive():
    # one hidden unit with a bias large enough to keep it positive: s = w2 (w.h + b1) + b2
    rng = np.random.default_rng(71)
    d = 16
    hb = f32_to_bf16_bits(rng.standard_normal((6, d)))
    w = rng.standard_normal(d).astype(np.float32)
    wb = f32_to_bf16_bits(w)[None, :]
    s, q = O.score_mlp(hb, wb, np.array([64.0], np.float32), np.array([0.5], np.float32), -32.0)
    w_rounded = O.bf16_bits_to_f64(wb[0]).astype(np.float32)
    s_lin, q_lin = O.score(hb, w_rounded, 0.0)
    assert np.allclose(s, 0.5 * s_lin, rtol=0, atol=1e-12) and np.allclose(q, 0.5 * (1 + np.tanh(0.25 * s_lin)), atol=1e-12)


def test_score_mlp_dead_units_and_unit_permutation():
    rng = np.random.default_rng(72)
    d, m, N = 8, 12, 5
    hb = f32_to_bf16_bits(rng.standard_normal((N, d)))
    W1 = f32_to_bf16_bits(rng.standard_normal((m, d)))
    b1 = rng.standard_normal(m).astype(np.float32)
    w2 = rng.standard_normal(m).astype(np.float32)
    s, q = O.score_mlp(hb, W1, b1, w2, 0.25)
    # every unit switched off by a very negative bias: only b2 is left
    s0, q0 = O.score_mlp(hb, W1, np.full(m, -1e6, np.float32), w2, 0.25)
    assert np.all(s0 == 0.25) and np.allclose(q0, 1 / (1 + math.exp(-0.25)), atol=1e-15)
    # hidden units are exchangeable
    perm = rng.permutation(m)
    s1, _ = O.score_mlp(hb, W1[perm], b1[perm], w2[perm], 0.25)
    assert np.allclose(s1, s, rtol=0, atol=1e-12)
    # s - b2 is linear in w2
    s2, _ = O.score_mlp(hb, W1, b1, (2 * w2).astype(np.float32), 0.25)
    assert np.allclose(s2 - 0.25, 2 * (s - 0.25), rtol=0, atol=1e-12)


def test_score_mlp_exact_rational():
    rng = np.random.default_rng(73)
    d, m = 6, 4
    hb = f32_to_bf16_bits(rng.standard_normal((3, d)))
    W1 = f32_to_bf16_bits(rng.standard_normal((m, d)))
    b1 = rng.standard_normal(m).astype(np.float32)
    w2 = rng.standard_normal(m).astype(np.float32)
    s, _ = O.score_mlp(hb, W1, b1, w2, -0.5)
    for i in range(3):
        tot = Fraction(-1, 2)
        for u in range(m):
            pre = sum(bits_to_fraction(W1[u, k]) * bits_to_fraction(hb[i, k]) for k in range(d)) + Fraction(float(b1[u]))
            if pre > 0:
                tot += pre * Fraction(float(w2[u]))
        assert abs(s[i] - float(tot)) < 1e-13


# ----------------------------------------------------------------------------- head training
def _head_case(seed, n=24, d=16, scale=0.5):
    rng = np.random.default_rng(seed)
    hb = f32_to_bf16_bits(rng.normal(size=(n, d)).astype(np.float32))
    w = (rng.normal(size=d) * scale).astype(np.float32)
    y = (rng.random(n) < 0.4).astype(np.float32)
    return hb, w, np.float32(rng.normal() * 0.3), y


def test_score_ce_at_zero_weights_is_ln2_and_gradient_is_the_label_offset():
    hb, w, _, y = _head_case(11)
    loss, gw, gb = O.score_ce_grad(hb, np.zeros_like(w), 0.0, y)
    assert abs(loss - math.log(2.0)) < 1e-15
    h = O.bf16_bits_to_f64(hb)
    assert np.allclose(gw, ((0.5 - y.astype(np.float64))[:, None] * h).mean(axis=0), rtol=0, atol=1e-15)
    assert abs(gb - float(np.mean(0.5 - y.astype(np.float64)))) < 1e-15


def test_score_ce_matches_the_definition_through_the_probabilities():
    # L = -mean(y log q + (1-y) log(1-q)) with q taken from the scoring oracle
    hb, w, b, y = _head_case(12)
    _, q = O.score(hb, w, b)
    y64 = y.astype(np.float64)
    direct = -np.mean(y64 * np.log(q) + (1.0 - y64) * np.log(1.0 - q))
    assert abs(O.score_ce(hb, w, b, y) - direct) < 1e-12


def test_score_ce_gradient_against_central_differences():
    hb, w, b, y = _head_case(13, n=20, d=8)
    loss, gw, gb = O.score_ce_grad(hb, w, b, y)
    assert abs(loss - O.score_ce(hb, w, b, y)) == 0.0
    # float32 parameters: step by whole fp32 increments so that w +- e is representable
    for c in range(8):
        e = np.float32(2.0 ** -7)
        wp, wm = w.copy(), w.copy()
        wp[c] = w[c] + e
        wm[c] = w[c] - e
        step = float(wp[c]) - float(wm[c])
        fd = (O.score_ce(hb, wp, b, y) - O.score_ce(hb, wm, b, y)) / step
        assert abs(fd - gw[c]) < 5e-5, (c, fd, gw[c])
    e = 2.0 ** -7
    fd = (O.score_ce(hb, w, float(b) + e, y) - O.score_ce(hb, w, float(b) - e, y)) / (2 * e)
    assert abs(fd - gb) < 5e-5


def test_score_ce_soft_labels_equal_to_the_prediction_have_zero_gradient():
    hb, w, b, _ = _head_case(14)
    _, q = O.score(hb, w, b)
    # labels are read as fp32, so the match is to fp32 rounding of q
    loss, gw, gb = O.score_ce_grad(hb, w, b, q.astype(np.float32))
    assert np.max(np.abs(gw)) < 1e-6 and abs(gb) < 1e-7
    # and the loss is then the mean binary entropy of q
    ent = -np.mean(q * np.log(q) + (1 - q) * np.log(1 - q))
    assert abs(loss - ent) < 1e-6


def test_score_ce_saturated_logits_stay_finite():
    hb = f32_to_bf16_bits(np.full((2, 8), 16.0, dtype=np.float32))
    w = np.full(8, 8.0, dtype=np.float32)                     # s = 1024
    loss, gw, gb = O.score_ce_grad(hb, w, 0.0, np.array([1.0, 0.0], dtype=np.float32))
    assert math.isfinite(loss) and abs(loss - 512.0) < 1e-9   # (0 + 1024)/2
    assert np.allclose(gw, 0.5 * 16.0) and abs(gb - 0.5) < 1e-12


def test_adamw_first_step_closed_form():
    # with zero state, m_hat = g and v_hat = g^2, so the step is lr*(g/(|g|+eps) + wd*p)
    p = np.array([1.0, -2.0, 0.5, 3.0], dtype=np.float32)
    g = np.array([0.25, -4.0, 0.0, 1e-3], dtype=np.float32)
    z = np.zeros(4, dtype=np.float32)
    p1, m1, v1 = O.adamw_step(p, g, z, z, 1, lr=0.1, beta1=0.9, beta2=0.99, eps=1e-8, weight_decay=0.01)
    g64, p64 = g.astype(np.float64), p.astype(np.float64)
    want = p64 - 0.1 * (g64 / (np.abs(g64) + 1e-8) + 0.01 * p64)
    assert np.allclose(p1, want, rtol=0, atol=1e-12)
    assert np.allclose(m1, 0.1 * g64, atol=1e-15) and np.allclose(v1, 0.01 * g64 * g64, atol=1e-15)


def test_adamw_matches_the_library_optimizer_over_several_steps():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    p0 = rng.normal(size=33).astype(np.float32)
    grads = [rng.normal(size=33).astype(np.float32) * (10.0 ** rng.integers(-3, 2)) for _ in range(6)]
    tp = torch.nn.Parameter(torch.tensor(p0, dtype=torch.float64))
    opt = torch.optim.AdamW([tp], lr=3e-2, betas=(0.8, 0.95), eps=1e-6, weight_decay=0.1)
    p = p0.astype(np.float64)
    m = np.zeros(33)
    v = np.zeros(33)
    for t, g in enumerate(grads, start=1):
        tp.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        p, m, v = O.adamw_step(p, g, m, v, t, 3e-2, 0.8, 0.95, 1e-6, 0.1)
        assert np.allclose(p, tp.detach().numpy(), rtol=1e-12, atol=1e-12), t


# ----------------------------------------------------------------------------- trace confidence
def test_token_confidence_uniform_distribution_is_V_ln_V_and_is_the_minimum():
    rng = np.random.default_rng(21)
    V, d = 37, 8
    Wb = f32_to_bf16_bits(rng.normal(size=(V, d)).astype(np.float32))
    zero_h = np.zeros((1, d), dtype=np.uint16)
    assert abs(O.token_confidence(zero_h, Wb)[0] - V * math.log(V)) < 1e-10
    # H_t / V - ln V is KL(uniform || P_t) >= 0
    hb = f32_to_bf16_bits(rng.normal(size=(6, d)).astype(np.float32))
    assert np.all(O.token_confidence(hb, Wb) > V * math.log(V))


def test_token_confidence_two_token_vocabulary_closed_form():
    # V = 2 with logits (a, b): H = log(1+e^{b-a}) + log(1+e^{a-b})
    Wb = f32_to_bf16_bits(np.array([[1.5, 0.0], [0.0, -0.75]], dtype=np.float32))
    hb = f32_to_bf16_bits(np.array([[2.0, 4.0], [-1.0, 0.5]], dtype=np.float32))
    got = O.token_confidence(hb, Wb)
    for t, (a, b) in enumerate([(3.0, -3.0), (-1.5, -0.375)]):
        want = math.log1p(math.exp(b - a)) + math.log1p(math.exp(a - b))
        assert abs(got[t] - want) < 1e-12


def test_token_confidence_equals_V_lse_minus_the_logit_sum_and_matches_logprob():
    rng = np.random.default_rng(22)
    V, d, T = 50, 16, 5
    Wb = f32_to_bf16_bits(rng.normal(size=(V, d)).astype(np.float32))
    hb = f32_to_bf16_bits(rng.normal(size=(T, d)).astype(np.float32))
    got = O.token_confidence(hb, Wb)
    z = O.bf16_bits_to_f64(hb) @ O.bf16_bits_to_f64(Wb).T
    _, lse = O.logprob(hb, Wb, np.zeros(T, dtype=np.int64))
    assert np.allclose(got, V * lse - z.sum(axis=1), rtol=1e-13)
    # summing the per-target log-probabilities over every target gives the same number
    total = np.zeros(T)
    for j in range(V):
        lp, _ = O.logprob(hb, Wb, np.full(T, j))
        total -= lp
    assert np.allclose(got, total, rtol=1e-13)


def test_trace_confidence_ramp_closed_forms():
    # conf_t = t on one trace of length 100, window 10: window k has mean k + 4.5, 91 windows,
    # bottom 10 % = ceil(9.1) = 10 lowest windows -> mean of 4.5 .. 13.5 = 9.0
    conf = np.arange(100, dtype=np.float64)
    mean, wmin, bottom = O.trace_confidence(conf, [0, 100], 10)
    assert mean[0] == 49.5 and wmin[0] == 4.5 and bottom[0] == 9.0
    # decreasing ramp: the lowest windows are the last ones
    mean, wmin, bottom = O.trace_confidence(conf[::-1].copy(), [0, 100], 10)
    assert mean[0] == 49.5 and wmin[0] == 4.5 and bottom[0] == 9.0


def test_trace_confidence_window_one_and_whole_trace_windows():
    rng = np.random.default_rng(23)
    conf = rng.normal(size=57) * 3 + 10
    mean, wmin, bottom = O.trace_confidence(conf, [0, 57], 1)
    srt = np.sort(conf)
    assert wmin[0] == srt[0] and abs(bottom[0] - srt[:6].mean()) < 1e-13     # ceil(5.7) = 6
    for w in (57, 58, 4096):
        mean, wmin, bottom = O.trace_confidence(conf, [0, 57], w)
        assert abs(mean[0] - conf.mean()) < 1e-13 and wmin[0] == mean[0] == bottom[0]


def test_trace_confidence_ragged_batch_empty_trace_and_exact_rational_brute_force():
    rng = np.random.default_rng(24)
    lens = [0, 1, 5, 12, 30, 3]
    cu = np.concatenate([[0], np.cumsum(lens)])
    conf = rng.integers(-50, 50, size=cu[-1]).astype(np.float64) / 4      # exact quarters
    w = 4
    mean, wmin, bottom = O.trace_confidence(conf, cu, w, bottom_percent=25)
    assert math.isnan(mean[0]) and math.isnan(wmin[0]) and math.isnan(bottom[0])
    for i, L in enumerate(lens):
        if L == 0:
            continue
        x = [Fraction(int(v * 4), 4) for v in conf[cu[i]:cu[i + 1]]]
        ww = min(w, L)
        wins = sorted(sum(x[k:k + ww], Fraction(0)) / ww for k in range(L - ww + 1))
        m = max(1, -(-len(wins) * 25 // 100))
        assert Fraction(mean[i]) == sum(x, Fraction(0)) / L or abs(mean[i] - float(sum(x, Fraction(0)) / L)) < 1e-14
        assert abs(wmin[i] - float(wins[0])) < 1e-14
        assert abs(bottom[i] - float(sum(wins[:m], Fraction(0)) / m)) < 1e-14


def test_trace_confidence_bottom_count_uses_integer_ceiling():
    # 30 windows at 10 % must take exactly 3 (a float product 0.1*30 rounds above 3)
    conf = np.arange(30, dtype=np.float64)
    _, _, bottom = O.trace_confidence(conf, [0, 30], 1)
    assert bottom[0] == 1.0          # mean of 0, 1, 2
    _, _, bottom = O.trace_confidence(np.arange(31, dtype=np.float64), [0, 31], 1)
    assert bottom[0] == 1.5          # ceil(3.1) = 4 -> mean of 0..3


# ----------------------------------------------------------------------------- GRPO
def test_grpo_advantage_binary_rewards_closed_form():
    # k ones among n: A(1) = sqrt((1-p)/p), A(0) = -sqrt(p/(1-p)) with p = k/n (population std)
    for n, k in [(4, 1), (8, 4), (16, 3), (5, 4)]:
        r = np.array([1.0] * k + [0.0] * (n - k), dtype=np.float32)
        adv = O.grpo_advantage(r, [0, n])
        p = k / n
        assert np.allclose(adv[:k], math.sqrt((1 - p) / p), rtol=1e-14)
        assert np.allclose(adv[k:], -math.sqrt(p / (1 - p)), rtol=1e-14)


def test_grpo_advantage_is_standardised_per_group_and_zero_for_equal_rewards():
    rng = np.random.default_rng(31)
    off = np.array([0, 4, 4, 9, 10, 26])            # an empty group and a singleton among them
    r = rng.normal(size=26).astype(np.float32)
    r[4:9] = 0.75                                   # all-equal group
    adv = O.grpo_advantage(r, off)
    for g in (0, 4):
        x = adv[off[g]:off[g + 1]]
        assert abs(x.mean()) < 1e-14 and abs(np.mean(x * x) - 1.0) < 1e-13
    assert np.all(adv[4:10] == 0.0)                 # equal rewards and the singleton
    # sample standard deviation (ddof = 1) rescales by sqrt((n-1)/n); eps enters the denominator
    a1 = O.grpo_advantage(r, off, ddof=1)
    assert np.allclose(a1[:4], adv[:4] * math.sqrt(3 / 4), rtol=1e-13)
    assert a1[9] == 0.0
    x = r[:4].astype(np.float64)
    ae = O.grpo_advantage(r, off, eps=0.5)
    assert np.allclose(ae[:4], (x - x.mean()) / (x.std() + 0.5), rtol=1e-13)


def test_grpo_objective_hand_worked_clipping_cases():
    # one group, four one-token rollouts: (r, A) = (2, 1), (2, -1), (0.5, 1), (0.5, -1), eps = 0.2
    lp = np.log(np.array([2.0, 2.0, 0.5, 0.5])).astype(np.float32)
    ratio = np.exp(lp.astype(np.float64))
    adv = np.array([1.0, -1.0, 1.0, -1.0], dtype=np.float32)
    J, grad, n_clip = O.grpo_objective(lp, np.zeros(4, dtype=np.float32), [0, 1, 2, 3, 4], adv, [0, 4])
    terms = [1.2, -ratio[1], ratio[2], -0.8]
    assert abs(J - sum(terms) / 4) < 1e-15
    assert n_clip == 2                               # the first and the last
    assert grad[0] == 0.0 and grad[3] == 0.0
    assert abs(grad[1] - (-ratio[1]) / 4) < 1e-15 and abs(grad[2] - ratio[2] / 4) < 1e-15


def test_grpo_objective_on_policy_is_the_mean_advantage_and_its_gradient():
    rng = np.random.default_rng(32)
    lens = [3, 5, 2, 4, 6, 1]
    cu = np.concatenate([[0], np.cumsum(lens)])
    off = [0, 2, 6]
    lp = (-rng.random(cu[-1]) * 3).astype(np.float32)
    r = rng.normal(size=6).astype(np.float32)
    adv = O.grpo_advantage(r, off).astype(np.float32)
    J, grad, n_clip = O.grpo_objective(lp, lp, cu, adv, off, beta=0.3)
    want = np.mean([adv[0:2].astype(np.float64).mean(), adv[2:6].astype(np.float64).mean()])
    assert abs(J - want) < 1e-15 and n_clip == 0    # ratio 1 everywhere, KL estimate 0
    for i, L in enumerate(lens):
        G = 2 if i < 2 else 4
        assert np.allclose(grad[cu[i]:cu[i + 1]], float(adv[i]) / (L * G * 2), rtol=1e-14)


def test_grpo_objective_gradient_against_central_differences():
    rng = np.random.default_rng(33)
    lens = [4, 3, 5, 2]
    cu = np.concatenate([[0], np.cumsum(lens)])
    off = [0, 2, 4]
    T = int(cu[-1])
    lr = (-rng.random(T) * 2).astype(np.float32)
    lp = (lr + rng.normal(size=T).astype(np.float32) * 0.3).astype(np.float32)
    adv = O.grpo_advantage(rng.normal(size=4).astype(np.float32), off).astype(np.float32)
    args = dict(eps_low=0.2, eps_high=0.28, beta=0.05)
    J, grad, n_clip = O.grpo_objective(lp, lr, cu, adv, off, **args)
    assert 0 < n_clip < T                           # both branches occur
    ratio = np.exp(lp.astype(np.float64) - lr)
    e = np.float32(2.0 ** -9)
    for t in range(T):
        if min(abs(ratio[t] - 0.8), abs(ratio[t] - 1.28)) < 0.01:
            continue                                # too close to a kink for a finite difference
        up, dn = lp.copy(), lp.copy()
        up[t] += e
        dn[t] -= e
        fd = (O.grpo_objective(up, lr, cu, adv, off, **args)[0] - O.grpo_objective(dn, lr, cu, adv, off, **args)[0]) \
            / (float(up[t]) - float(dn[t]))
        assert abs(fd - grad[t]) < 1e-5 * max(1.0, abs(grad[t]) * 100), (t, fd, grad[t])


def test_grpo_kl_estimate_is_nonnegative_and_unbiased_by_enumeration():
    # E_{x ~ p}[exp(u) - u - 1] with u = log q(x) - log p(x) equals KL(p || q), summed over a small alphabet
    rng = np.random.default_rng(34)
    p = rng.random(7); p /= p.sum()
    q = rng.random(7); q /= q.sum()
    lp, lq = np.log(p).astype(np.float32), np.log(q).astype(np.float32)
    # one rollout per symbol, one token each, advantage 0, beta 1: J = -(1/7) sum_x kl(x); weight by p by hand
    total = 0.0
    for x in range(7):
        J, _, _ = O.grpo_objective(lp[x:x + 1], lq[x:x + 1], [0, 1], np.zeros(1, dtype=np.float32), [0, 1], beta=1.0)
        assert J <= 0.0
        total += float(np.exp(np.float64(lp[x]))) * (-J)
    p32, q32 = np.exp(lp.astype(np.float64)), np.exp(lq.astype(np.float64))
    kl = float(np.sum(p32 * (np.log(p32) - np.log(q32)))) + float(np.sum(q32) - np.sum(p32))
    assert abs(total - kl) < 1e-12


# ----------------------------------------------------------------------------- MLP head training
def _mlp_case(seed, n=12, d=8, m=6):
    rng = np.random.default_rng(seed)
    hb = f32_to_bf16_bits(rng.normal(size=(n, d)).astype(np.float32))
    w1b = f32_to_bf16_bits((rng.normal(size=(m, d)) * 0.5).astype(np.float32))
    b1 = (rng.normal(size=m) * 0.2).astype(np.float32)
    w2 = (rng.normal(size=m) * 0.7).astype(np.float32)
    y = (rng.random(n) < 0.5).astype(np.float32)
    return hb, w1b, b1, w2, np.float32(0.1), y


def _mlp_loss(hb, w1b, b1, w2, b2, y):
    """Mean cross-entropy through the forward oracle's logits (definition, not the gradient routine)."""
    s, _ = O.score_mlp(hb, w1b, b1, w2, b2)
    y = y.astype(np.float64)
    return float(np.mean(np.maximum(s, 0) - y * s + np.log1p(np.exp(-np.abs(s)))))


def test_mlp_grad_loss_is_the_cross_entropy_of_the_forward_oracle():
    case = _mlp_case(41)
    loss = O.score_mlp_ce_grad(*case)[0]
    assert abs(loss - _mlp_loss(*case)) < 1e-13


def test_mlp_grad_against_central_differences_of_the_loss():
    hb, w1b, b1, w2, b2, y = _mlp_case(42)
    _, gW1, gb1, gw2, gb2 = O.score_mlp_ce_grad(hb, w1b, b1, w2, b2, y)
    e = 2.0 ** -10
    # fp32 parameters: perturb by an exactly representable step
    for u in range(6):
        for arr, g in ((b1, gb1), (w2, gw2)):
            up, dn = arr.copy(), arr.copy()
            up[u] += np.float32(e)
            dn[u] -= np.float32(e)
            a_up = (hb, w1b, up, w2, b2, y) if arr is b1 else (hb, w1b, b1, up, b2, y)
            a_dn = (hb, w1b, dn, w2, b2, y) if arr is b1 else (hb, w1b, b1, dn, b2, y)
            fd = (_mlp_loss(*a_up) - _mlp_loss(*a_dn)) / (float(up[u]) - float(dn[u]))
            assert abs(fd - g[u]) < 1e-6, (u, fd, g[u])
    fd = (_mlp_loss(hb, w1b, b1, w2, np.float32(b2 + e), y) - _mlp_loss(hb, w1b, b1, w2, np.float32(b2 - e), y)) \
        / (float(np.float32(b2 + e)) - float(np.float32(b2 - e)))
    assert abs(fd - gb2) < 1e-6
    # W1 is bf16: step to the neighbouring representable values (one ulp each way)
    W1 = O.bf16_bits_to_f64(w1b)
    for (u, c) in [(0, 0), (2, 5), (5, 7), (3, 3)]:
        up, dn = w1b.copy(), w1b.copy()
        sign_neg = bool(w1b[u, c] >> 15)
        up[u, c] = int(w1b[u, c]) + (-1 if sign_neg else 1)
        dn[u, c] = int(w1b[u, c]) + (1 if sign_neg else -1)
        step = O.bf16_bits_to_f64(up)[u, c] - O.bf16_bits_to_f64(dn)[u, c]
        assert step > 0
        fd = (_mlp_loss(hb, up, b1, w2, b2, y) - _mlp_loss(hb, dn, b1, w2, b2, y)) / step
        # a one-ulp bf16 step is coarse (2^-8 relative): allow the second-order term, and skip kinks
        pre_up = O.bf16_bits_to_f64(up) @ O.bf16_bits_to_f64(hb).T + b1[:, None]
        pre_dn = O.bf16_bits_to_f64(dn) @ O.bf16_bits_to_f64(hb).T + b1[:, None]
        if np.any((pre_up > 0) != (pre_dn > 0)):
            continue
        assert abs(fd - gW1[u, c]) < 2e-3 * max(1e-2, abs(gW1[u, c])), (u, c, fd, gW1[u, c])


def test_mlp_grad_reduces_to_the_linear_head_when_every_unit_is_active():
    # large positive b1 keeps every pre-activation positive: s = <W1^T w2, h> + (<w2, b1> + b2), so the
    # gradients follow from the linear head's by the chain rule
    rng = np.random.default_rng(43)
    n, d, m = 10, 8, 4
    hb = f32_to_bf16_bits(rng.normal(size=(n, d)).astype(np.float32))
    w1b = f32_to_bf16_bits((rng.normal(size=(m, d)) * 0.25).astype(np.float32))
    b1 = np.full(m, 64.0, dtype=np.float32)
    w2 = np.array([0.5, -0.25, 0.125, -0.5], dtype=np.float32)      # exact in fp32, keeps w_eff representable
    b2 = np.float32(0.0)
    y = (rng.random(n) < 0.5).astype(np.float32)
    W1 = O.bf16_bits_to_f64(w1b)
    w_eff = W1.T @ w2.astype(np.float64)
    bias_eff = float(np.dot(w2.astype(np.float64), b1.astype(np.float64)))
    assert np.all(w_eff.astype(np.float32).astype(np.float64) == w_eff)
    loss_lin, gw_lin, gb_lin = O.score_ce_grad(hb, w_eff.astype(np.float32), bias_eff, y)
    loss, gW1, gb1, gw2, gb2 = O.score_mlp_ce_grad(hb, w1b, b1, w2, b2, y)
    assert abs(loss - loss_lin) < 1e-13
    assert np.allclose(gW1, np.outer(w2.astype(np.float64), gw_lin), rtol=1e-12, atol=1e-15)
    assert np.allclose(gb1, w2.astype(np.float64) * gb_lin, rtol=1e-12, atol=1e-15)
    assert abs(gb2 - gb_lin) < 1e-15
    # dL/dw2 = sum_i r_i (W1 h_i + b1) = W1 gw_lin + b1 gb_lin
    assert np.allclose(gw2, W1 @ gw_lin + b1.astype(np.float64) * gb_lin, rtol=1e-12, atol=1e-14)


def test_mlp_grad_dead_units_get_no_gradient():
    hb, w1b, b1, w2, b2, y = _mlp_case(44)
    b1 = b1.copy()
    b1[1] = -1000.0                                   # unit 1 never fires
    _, gW1, gb1, gw2, _ = O.score_mlp_ce_grad(hb, w1b, b1, w2, b2, y)
    assert np.all(gW1[1] == 0.0) and gb1[1] == 0.0 and gw2[1] == 0.0
    assert np.any(gW1[0] != 0.0)


def test_grpo_objective_asymmetric_clip_range_hand_worked():
    # eps_low = 0.1, eps_high = 0.3 (DAPO-style clip-higher): the range is [0.9, 1.3]
    ratios = np.array([1.25, 1.5, 0.85, 0.95])
    lp = np.log(ratios).astype(np.float32)
    ratio = np.exp(lp.astype(np.float64))
    adv = np.array([1.0, 1.0, -1.0, -1.0], dtype=np.float32)
    e_lo, e_hi = float(np.float32(0.1)), float(np.float32(0.3))
    J, grad, n_clip = O.grpo_objective(lp, np.zeros(4, dtype=np.float32), [0, 1, 2, 3, 4], adv, [0, 4],
                                       eps_low=e_lo, eps_high=e_hi)
    # 1.25 inside the range; 1.5 clipped at 1 + eps_high; 0.85 with A < 0: min(-0.85, -(1 - eps_low)) = -(1 - eps_low);
    # 0.95 inside
    terms = [ratio[0], 1.0 + e_hi, -(1.0 - e_lo), -ratio[3]]
    assert abs(J - sum(terms) / 4) < 1e-15
    assert n_clip == 2 and grad[1] == 0.0 and grad[2] == 0.0
