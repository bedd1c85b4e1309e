"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: every configuration
(LLaMA-3.2-1B-, Qwen3-1.7B-, LLaMA-3.2-3B- and Qwen3-8B-shaped batches) on sampled outputs the oracle
computes one by one - log-probs on a seeded row sample that always holds the edge rows, compaction byte
for byte on the first, a middle and the last KV layer plus a gather property on every layer - and
reduced-batch cases with the same geometries (ragged pools with spare pages)."""
import numpy as np
import pytest
import torch

import oracle as O
from helpers import bits, npy, to_dev, oracle_survivors

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def A():
    import paper_2603_24840_amd as pkg
    pkg.lib()
    return pkg


@pytest.fixture(scope="module")
def W():
    from paper_2603_24840_amd import workloads
    return workloads


def say(msg):
    print("[case] " + msg, flush=True)


def sample_rows(T, n, V, targets, seed=7, cu=None):
    """Seeded row sample that always holds the first / last rows, the first and last row of the first and last
    survivor, and rows whose target sits on a vocabulary-tile edge or at the ends of the vocabulary (the
    input generator plants such targets; any other row that happens to carry one is added too)."""
    from paper_2603_24840_amd.workloads import logprob_check_rows
    rows = set(logprob_check_rows(T, n, V, cu, seed).tolist())
    t = npy(targets)
    last_edge = (V - 1) // 256 * 256
    for want in (0, V - 1, 255, 256, last_edge - 1, last_edge):
        hit = np.flatnonzero(t == want)
        if hit.size:
            rows.add(int(hit[0]))
    return torch.tensor(sorted(rows), dtype=torch.int64)


def free():
    import gc
    gc.collect()
    torch.cuda.empty_cache()


def test_llama1b_prune_path_full_size(A, W):
    cfg = W.CONFIGS["llama1b"]
    say("llama1b score/select/vote, full batch")
    hidden, w, b = W.score_inputs(cfg, DEV)
    s, q = A.arrol_score(hidden, w, b)
    keep, surv = A.arrol_select(q, cfg.n_prompts, cfg.G, cfg.K, cfg.rho)
    _, ans = W.vote_inputs(cfg, DEV)
    win, tally = A.arrol_weighted_vote(q, ans, cfg.vote_q, cfg.vote_c, cfg.vote_a, want_tally=True)
    torch.cuda.synchronize()
    so, qo = O.score(bits(hidden), npy(w), b)
    assert np.max(np.abs(npy(q) - qo)) < 1e-3 and np.max(np.abs(npy(s) - so)) < 1e-3
    # the oracle's chain runs from the inputs alone; the library is checked on the oracle's probabilities
    # (stage parity) and on its own (chain parity: rounding-level differences, no tie that close here)
    q32 = qo.astype(np.float32)
    keep_o, surv_o = oracle_survivors(O, q32, cfg)
    win_o, tally_o = O.weighted_vote(q32, npy(ans), cfg.vote_q, cfg.vote_c, cfg.vote_a)
    keep2, surv2 = A.arrol_select(to_dev(q32, DEV), cfg.n_prompts, cfg.G, cfg.K, cfg.rho)
    win2, tally2 = A.arrol_weighted_vote(to_dev(q32, DEV), ans, cfg.vote_q, cfg.vote_c, cfg.vote_a, want_tally=True)
    torch.cuda.synchronize()
    assert np.array_equal(npy(keep2), keep_o) and np.array_equal(npy(surv2), surv_o)
    assert np.array_equal(npy(win2), win_o) and np.array_equal(npy(tally2), tally_o)
    assert np.array_equal(npy(keep), keep_o) and np.array_equal(npy(surv), surv_o)
    assert np.array_equal(npy(win), win_o) and np.array_equal(npy(tally), tally_o)


def test_llama1b_compact_full_size(A, W):
    cfg = W.CONFIGS["llama1b"]
    say("llama1b compact, full pool (8.6 GB), oracle on 4 of 16 layers + gather property on all")
    kv, bt, sl, tok = W.compact_inputs(cfg, DEV)
    p = W.select_inputs(cfg, DEV)                                  # seeded probabilities (an input)
    _, surv_o = oracle_survivors(O, npy(p), cfg)
    _, surv = A.arrol_select(p, cfg.n_prompts, cfg.G, cfg.K, cfg.rho)
    torch.cuda.synchronize()
    assert np.array_equal(npy(surv), surv_o)
    n_dst = cfg.n_keep * cfg.pages_per_rollout
    dst = torch.empty((cfg.n_layers, 2, n_dst) + tuple(kv.shape[3:]), dtype=torch.bfloat16, device=DEV)
    dst.view(torch.int16).fill_(0x7FC1)
    out = A.arrol_compact(kv, dst, bt, sl, tok, surv)
    torch.cuda.synchronize()
    surv_h, bt_h, sl_h, tok_h = surv_o, npy(bt), npy(sl), npy(tok)
    for layer in (0, 5, 10, cfg.n_layers - 1):
        ref = O.compact(bits(kv[layer:layer + 1]), bt_h, sl_h, tok_h, surv_h, n_dst, fill=0x7FC1)
        assert np.array_equal(bits(dst[layer:layer + 1]), ref["kv_dst"]), layer
    assert np.array_equal(npy(out["block_table_dst"]), ref["block_table_dst"])
    assert np.array_equal(npy(out["tokens_dst"]), ref["tokens_dst"])
    assert np.array_equal(npy(out["seq_len_dst"]), ref["seq_len_dst"])
    assert np.array_equal(npy(out["src_of_dst"]), ref["src_of_dst"])
    assert int(out["n_pages_used"][0]) == ref["n_pages_used"] == n_dst
    # every layer: destination page j holds source page flat[j]  (holds at any size)
    flat = bt[surv.long()].reshape(-1).long()
    for layer in range(cfg.n_layers):
        for c in range(2):
            assert torch.equal(dst[layer, c].view(torch.int16), kv[layer, c, flat].view(torch.int16)), (layer, c)


def test_llama1b_logprob_full_size_sampled_rows(A, W):
    cfg = W.CONFIGS["llama1b"]
    say("llama1b logprob, full T x V x d, 160 sampled rows against the oracle")
    hidden, lm_head, targets, cu = W.logprob_inputs(cfg, DEV)
    T = hidden.shape[0]
    assert 256 * cfg.n_keep <= T <= 2048 * cfg.n_keep and lm_head.shape == (128256, 2048)
    lp, lse = A.arrol_logprob(hidden, lm_head, targets, want_lse=True)
    torch.cuda.synchronize()
    rows = sample_rows(T, 150, cfg.vocab, targets, cu=cu)
    lp_o, lse_o = O.logprob(bits(hidden[rows.to(DEV)]), bits(lm_head), npy(targets)[rows.numpy()])
    assert np.max(np.abs(npy(lp)[rows.numpy()] - lp_o)) < 1e-4      # the bar is 2e-3; 1e-4 is what fp32 accumulation allows here
    assert np.max(np.abs(npy(lse)[rows.numpy()] - lse_o)) < 1e-4
    # whole output: finite, negative, and distributed as logits ~ N(0,1) imply (lse ~ log V + 1/2)
    assert bool(torch.isfinite(lp).all()) and float(lp.max()) <= 0.0
    assert abs(float(lse.mean()) - (np.log(cfg.vocab) + 0.5)) < 0.05


BIG = ["qwen1p7b", "llama3b", "qwen8b"]


@pytest.mark.parametrize("name", BIG)
def test_prune_and_compact_full_size(A, W, name):
    """score -> select -> compact on the whole batch and the whole KV pool (120-155 GB source, 60-77 GB
    destination): the library's chain against the oracle's chain from the same seeded inputs."""
    cfg = W.CONFIGS[name]
    say("%s score/select/vote full batch, then compact of the full pool" % name)
    free()
    hidden, w, b = W.score_inputs(cfg, DEV)
    s, q = A.arrol_score(hidden, w, b)
    keep, surv = A.arrol_select(q, cfg.n_prompts, cfg.G, cfg.K, cfg.rho)
    torch.cuda.synchronize()
    so, qo = O.score(bits(hidden), npy(w), b)
    assert np.max(np.abs(npy(q) - qo)) < 1e-3 and np.max(np.abs(npy(s) - so)) < 1e-3
    q32 = qo.astype(np.float32)
    keep_o, surv_o = oracle_survivors(O, q32, cfg)
    keep2, surv2 = A.arrol_select(to_dev(q32, DEV), cfg.n_prompts, cfg.G, cfg.K, cfg.rho)
    torch.cuda.synchronize()
    assert np.array_equal(npy(keep2), keep_o) and np.array_equal(npy(surv2), surv_o)     # stage parity
    assert np.array_equal(npy(keep), keep_o) and np.array_equal(npy(surv), surv_o)       # chain parity
    if cfg.vote_q * cfg.vote_c <= cfg.n_rollouts:       # the benchmark votes on the batch's own probabilities
        _, ans = W.vote_inputs(cfg, DEV)
        n = cfg.vote_q * cfg.vote_c
        win, tally = A.arrol_weighted_vote(q[:n].contiguous(), ans, cfg.vote_q, cfg.vote_c, cfg.vote_a, want_tally=True)
        torch.cuda.synchronize()
        win_o, tally_o = O.weighted_vote(q32[:n], npy(ans), cfg.vote_q, cfg.vote_c, cfg.vote_a)
        assert np.array_equal(npy(win), win_o) and np.array_equal(npy(tally), tally_o)
    del hidden
    say("%s pool: %d pages x %d layers" % (name, cfg.n_rollouts * cfg.pages_per_rollout, cfg.n_layers))
    kv, bt, sl, tok = W.compact_inputs(cfg, DEV)
    n_dst = cfg.n_keep * cfg.pages_per_rollout
    dst = torch.empty((cfg.n_layers, 2, n_dst) + tuple(kv.shape[3:]), dtype=torch.bfloat16, device=DEV)
    for layer in range(cfg.n_layers):                   # NaN pattern: a page the call skips stays visible
        dst[layer].view(torch.int16).fill_(0x7FC1)
    out = A.arrol_compact(kv, dst, bt, sl, tok, surv)
    torch.cuda.synchronize()
    say("%s compact done; oracle on layers 0, %d, %d" % (name, cfg.n_layers // 2, cfg.n_layers - 1))
    bt_h, sl_h, tok_h = npy(bt), npy(sl), npy(tok)
    ref = None
    for layer in (0, cfg.n_layers // 2, cfg.n_layers - 1):
        ref = O.compact(bits(kv[layer:layer + 1]), bt_h, sl_h, tok_h, surv_o, n_dst, fill=0x7FC1)
        assert np.array_equal(bits(dst[layer:layer + 1]), ref["kv_dst"]), layer
        say("%s layer %d bit-exact" % (name, layer))
    assert np.array_equal(npy(out["block_table_dst"]), ref["block_table_dst"])
    assert np.array_equal(npy(out["tokens_dst"]), ref["tokens_dst"])
    assert np.array_equal(npy(out["seq_len_dst"]), ref["seq_len_dst"])
    assert np.array_equal(npy(out["src_of_dst"]), ref["src_of_dst"])
    assert int(out["n_pages_used"][0]) == ref["n_pages_used"] == n_dst
    del ref
    # every layer: destination page j holds source page flat[j]  (holds at any size)
    flat = bt[surv.long()].reshape(-1).long()
    for layer in range(cfg.n_layers):
        for c in range(2):
            assert torch.equal(dst[layer, c].view(torch.int16), kv[layer, c].view(torch.int16)[flat]), (layer, c)
    del kv, dst, flat
    free()


@pytest.mark.parametrize("name", BIG)
def test_logprob_full_size_sampled_rows(A, W, name):
    """The fused log-prob pass over the configuration's full T x V x d (1.2-2.4 M response tokens), with
    more than 1,024 rows checked against the float64 oracle, edge rows and edge targets among them."""
    cfg = W.CONFIGS[name]
    free()
    hidden, lm_head, targets, cu = W.logprob_inputs(cfg, DEV)
    T = hidden.shape[0]
    say("%s logprob full size: T=%d V=%d d=%d" % (name, T, cfg.vocab, cfg.d))
    assert cfg.resp_lo * cfg.n_keep <= T <= cfg.resp_hi * cfg.n_keep and lm_head.shape == (cfg.vocab, cfg.d)
    lp, lse = A.arrol_logprob(hidden, lm_head, targets, want_lse=True)
    torch.cuda.synchronize()
    rows = sample_rows(T, 1024, cfg.vocab, targets, cu=cu)
    must = {0, T - 1, int(cu[1]) - 1, int(cu[-2]), int(cu[-1]) - 1} | {r for r, _ in W.edge_target_rows(T, cfg.vocab)}
    assert must <= set(rows.tolist()) and len(rows) >= 1024
    t_s = npy(targets)[rows.numpy()]
    last_edge = (cfg.vocab - 1) // 256 * 256
    assert {0, cfg.vocab - 1, 255, 256, last_edge - 1, last_edge} <= set(t_s.tolist())
    say("%s oracle on %d rows" % (name, len(rows)))
    lp_o, lse_o = O.logprob(bits(hidden[rows.to(DEV)]), bits(lm_head), t_s)
    assert np.max(np.abs(npy(lp)[rows.numpy()] - lp_o)) < 1e-4      # the bar is 2e-3; 1e-4 is what fp32 accumulation allows here
    assert np.max(np.abs(npy(lse)[rows.numpy()] - lse_o)) < 1e-4
    # whole output: finite, negative, and distributed as logits ~ N(0,1) imply (lse ~ log V + 1/2)
    assert bool(torch.isfinite(lp).all()) and float(lp.max()) <= 0.0
    assert abs(float(lse.mean()) - (np.log(cfg.vocab) + 0.5)) < 0.05
    # every sum is taken in a fixed order: a second pass gives the same bits on all T rows (a workgroup that read an
    # LDS slot before its loads had landed, or after it was refilled, would show up here)
    lp2, lse2 = A.arrol_logprob(hidden, lm_head, targets, want_lse=True)
    torch.cuda.synchronize()
    assert torch.equal(lp, lp2) and torch.equal(lse, lse2)
    del hidden, lm_head, lp, lse, lp2, lse2
    free()


@pytest.mark.parametrize("name,T", [("qwen1p7b", 300), ("llama3b", 257), ("qwen8b", 200)])
def test_logprob_other_model_geometries(A, W, name, T):
    cfg = W.CONFIGS[name]
    say("logprob %s geometry: V=%d d=%d, T=%d" % (name, cfg.vocab, cfg.d, T))
    hidden, lm_head, targets, _ = W.logprob_inputs(cfg, DEV, T=T)
    targets[0] = cfg.vocab - 1; targets[1] = 0; targets[2] = (cfg.vocab // 256) * 256 - 1
    lp = A.arrol_logprob(hidden, lm_head, targets)
    torch.cuda.synchronize()
    rows = sample_rows(T, 40, cfg.vocab, targets)
    lp_o, _ = O.logprob(bits(hidden[rows.to(DEV)]), bits(lm_head), npy(targets)[rows.numpy()])
    assert np.max(np.abs(npy(lp)[rows.numpy()] - lp_o)) < 1e-4
    assert bool(torch.isfinite(lp).all())


@pytest.mark.parametrize("name", ["qwen1p7b", "llama3b", "qwen8b"])
def test_prune_path_other_model_geometries(A, W, name):
    full = W.CONFIGS[name]
    cfg = W.shrink(full, n_prompts=6, n_layers=3)          # same d, G, K, head_dim, page size, checkpoint length
    say("prune path %s geometry: G=%d K=%d d=%d hd=%d, %d prompts, %d layers"
        % (name, cfg.G, cfg.K, cfg.d, cfg.head_dim, cfg.n_prompts, cfg.n_layers))
    hidden, w, b = W.score_inputs(cfg, DEV)
    kv, bt, sl, tok = W.compact_inputs(cfg, DEV, extra_pages=9)
    _, q = A.arrol_score(hidden, w, b)
    keep, surv = A.arrol_select(q, cfg.n_prompts, cfg.G, cfg.K, cfg.rho)
    n_dst = cfg.n_keep * cfg.pages_per_rollout
    dst = torch.zeros((cfg.n_layers, 2, n_dst) + tuple(kv.shape[3:]), dtype=torch.bfloat16, device=DEV)
    out = A.arrol_compact(kv, dst, bt, sl, tok, surv)
    torch.cuda.synchronize()
    _, qo = O.score(bits(hidden), npy(w), b)
    assert np.max(np.abs(npy(q) - qo)) < 1e-3
    q32 = qo.astype(np.float32)
    keep_o, surv_o = oracle_survivors(O, q32, cfg)
    keep2, surv2 = A.arrol_select(to_dev(q32, DEV), cfg.n_prompts, cfg.G, cfg.K, cfg.rho)
    assert np.array_equal(npy(keep2), keep_o) and np.array_equal(npy(surv2), surv_o)     # stage parity
    assert np.array_equal(npy(keep), keep_o) and np.array_equal(npy(surv), surv_o)       # chain parity
    ref = O.compact(bits(kv), npy(bt), npy(sl), npy(tok), surv_o, n_dst)
    assert np.array_equal(bits(dst), ref["kv_dst"])
    assert np.array_equal(npy(out["block_table_dst"]), ref["block_table_dst"])
    assert np.array_equal(npy(out["tokens_dst"]), ref["tokens_dst"])


def test_vote_test_time_shape_qwen8b(A, W):
    cfg = W.CONFIGS["qwen8b"]
    say("test-time scaling shape: %d questions x %d candidates, d=%d" % (cfg.vote_q, cfg.vote_c, cfg.d))
    hidden, ans = W.vote_inputs(cfg, DEV)
    _, w, b = W.score_inputs(cfg, DEV, n_rows=1)
    _, q = A.arrol_score(hidden, w, b)
    win, tally = A.arrol_weighted_vote(q, ans, cfg.vote_q, cfg.vote_c, cfg.vote_a, want_tally=True)
    torch.cuda.synchronize()
    rows = np.arange(0, hidden.shape[0], 97)
    _, qo = O.score(bits(hidden[torch.from_numpy(rows).to(DEV)]), npy(w), b)
    assert np.max(np.abs(npy(q)[rows] - qo)) < 1e-3
    # the vote at this shape on seeded probabilities (inputs, with exact ties among them) against the oracle
    g = torch.Generator(device=DEV); g.manual_seed(88)
    p = (torch.randint(0, 4096, (hidden.shape[0],), generator=g, device=DEV).float() / 4096.0).contiguous()
    win2, tally2 = A.arrol_weighted_vote(p, ans, cfg.vote_q, cfg.vote_c, cfg.vote_a, want_tally=True)
    torch.cuda.synchronize()
    win_o, tally_o = O.weighted_vote(npy(p), npy(ans), cfg.vote_q, cfg.vote_c, cfg.vote_a)
    assert np.array_equal(npy(win2), win_o) and np.array_equal(npy(tally2), tally_o)
    # the chain's vote (library scores -> library vote): every question has a winner among its candidates' answers
    a = npy(ans).reshape(cfg.vote_q, cfg.vote_c)
    wn = npy(win)
    assert all(wn[i] in a[i] for i in range(cfg.vote_q))
    assert np.array_equal(npy(tally).sum(axis=1), np.full(cfg.vote_q, cfg.vote_c * (cfg.vote_c - 1), dtype=np.int64))
