"""Benchmark of the ARRoL pruning path on one MI355X.

A step is one pass of the whole hot path over one synthetic batch:
  arrol_score -> arrol_select -> arrol_compact -> arrol_logprob -> arrol_weighted_vote
all enqueued on one stream with no host synchronisation in between.  Inputs are resident in
HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama1b] [--skip-cpu-baseline]
  python bench.py --calibrate-copy      # plain 1 GiB device copy, for scaling rocprof byte counters
  python bench.py --extras              # adds timings of the calls outside the five-stage step
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak, published

# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs scaled by the plain-copy calibration (profiles/); None where not measured.
PROFILED_TRAFFIC_BYTES = {
    ("llama1b", "logprob"): 2.7727e11,   # profiles/hbm_traffic_llama1b.txt (fabric-level fetch incl. Infinity-Cache hits)
    ("llama1b", "compact"): 8.593e9,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="llama1b")
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-rows", type=int, default=24576)
    ap.add_argument("--calibrate-copy", action="store_true")
    ap.add_argument("--inplace-compaction", action="store_true",
                    help="also time arrol_compact_inplace on the same pool and survivors (extra JSON object)")
    ap.add_argument("--extras", action="store_true",
                    help="also time the entry points outside the five-stage step (stochastic policy, MLP head, head "
                         "training, trace confidence, GRPO objective) on the same workload (extra JSON object)")
    ap.add_argument("--tune", default="", help="comma list key=value passed to arrol_set_tuning (experiments)")
    ap.add_argument("--only", default="", help="comma list of stages to run (profiling aid); default all")
    return ap.parse_args()


def calibrate_copy(torch):
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda:0").random_(0, 255)
    dst = torch.empty_like(src)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for _ in range(3):
        dst.copy_(src)
    ev[0].record()
    for _ in range(10):
        dst.copy_(src)
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / 10
    print(json.dumps({"calibrate_copy_bytes_read": n, "calibrate_copy_bytes_written": n, "ms": ms,
                      "GBps_read_plus_write": 2 * n / ms / 1e6}))


def cpu_baseline(cfg, t, sample_rows, torch):
    """The oracle, as it stands, timed on this machine's host cores on a bounded sample of the same
    step; per-stage times are scaled to the full step."""
    import numpy as np
    import oracle as O
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from helpers import bits, npy

    cores = torch.get_num_threads()
    T = t["lp_hidden"].shape[0]
    times = {}
    t0 = time.perf_counter()
    _, q = O.score(bits(t["hidden"]), npy(t["w"]), t["bias"])
    times["score"] = time.perf_counter() - t0
    q32 = q.astype(np.float32)            # the oracle's own chain: its probabilities at the interface precision
    t0 = time.perf_counter()
    _, surv = O.select(q32, cfg.n_prompts, cfg.G, cfg.K, cfg.rho)
    times["select"] = time.perf_counter() - t0
    select_ok = bool(np.array_equal(npy(t["surv"]), surv))
    # compact: two layers of the pool, scaled to all layers (layers are independent slabs)
    L_s = min(2, cfg.n_layers)
    kv_host = bits(t["kv_src"][:L_s])
    bt, sl, tok = npy(t["block_table"]), npy(t["seq_len"]), npy(t["tokens"])
    t0 = time.perf_counter()
    ref = O.compact(kv_host, bt, sl, tok, surv, t["kv_dst"].shape[2])
    times["compact"] = (time.perf_counter() - t0) * cfg.n_layers / L_s
    compact_ok = bool(np.array_equal(bits(t["kv_dst"][:L_s]), ref["kv_dst"]))
    del kv_host, ref
    # logprob: a seeded sample of rows (always row 0 and row T-1)
    g = torch.Generator(device="cpu"); g.manual_seed(12345)
    rows = torch.randperm(T, generator=g)[:max(2, min(sample_rows, T))]
    rows[0], rows[1] = 0, T - 1
    rows = torch.sort(rows)[0]
    h_s = bits(t["lp_hidden"][rows.to(t["lp_hidden"].device)])
    w_b = bits(t["lm_head"])
    y_s = npy(t["targets"])[rows.numpy()]
    t0 = time.perf_counter()
    lp_o, _ = O.logprob(h_s, w_b, y_s)
    dt = time.perf_counter() - t0
    times["logprob"] = dt * T / len(rows)
    err = float(np.max(np.abs(npy(t["logprob"])[rows.numpy()].astype(np.float64) - lp_o)))
    t0 = time.perf_counter()
    if t["vote_hidden"] is None:            # the vote ran on the batch's own probabilities
        vote_q32 = q32[:cfg.vote_q * cfg.vote_c]
    else:                                   # test-time shape: the vote stage scored its own candidates
        vote_q32 = O.score(bits(t["vote_hidden"]), npy(t["w"]), t["bias"])[1].astype(np.float32)
    O.weighted_vote(vote_q32, npy(t["answer_id"]), cfg.vote_q, cfg.vote_c, cfg.vote_a)
    times["vote"] = time.perf_counter() - t0
    total = sum(times.values())
    return {"value": T / total, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": "score/select/vote on the full batch; compact on %d of %d layers; logprob on %d of %d "
                      "rows (seeded, incl. first and last); stage times scaled to the full step"
                      % (L_s, cfg.n_layers, len(rows), T),
            "stage_seconds_scaled": {k: round(v, 4) for k, v in times.items()},
            "parity_on_sample": {"logprob_max_abs_err": err, "select_identical": select_ok,
                                 "compact_bit_exact": compact_ok}}


def time_score_test_time_shape(A, W, dev, torch, reps=10):
    """arrol_score at the test-time-scaling shape of the largest configuration (512 questions x 64 candidates,
    d = 4096): the one shape at which scoring is bandwidth- rather than launch-bound."""
    big = W.CONFIGS["qwen8b"]
    n_big = big.vote_q * big.vote_c
    gb = torch.Generator(device=dev); gb.manual_seed(5)
    h_big = W.randn_bf16((n_big, big.d), gb, dev)
    w_big = torch.randn(big.d, generator=gb, device=dev) * big.d ** -0.5
    s_big = torch.empty(n_big, device=dev)
    q_big = torch.empty(n_big, device=dev)
    run = lambda: A.arrol_score(h_big, w_big, 0.0, out_score=s_big, out_prob=q_big)
    for _ in range(2):
        run()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    by = n_big * big.d * 2.0 + big.d * 4.0 + n_big * 8.0
    return {"bound": "hbm", "kernel": "score_reg_kernel at N=%d, d=%d (test-time scaling shape)" % (n_big, big.d),
            "achieved": by / ms / 1e6, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": by / ms / 1e6 / HBM_PEAK_GBPS,
            "ms": ms}


def time_extras(A, W, cfg, dev, torch, lp_hidden, lm_head, targets, cu, lws, reps=10):
    """HIP-event timings of the calls that are not part of the five-stage step, at this workload's shapes.
    Each figure is the mean over `reps` back-to-back calls after two warm-up calls."""
    def timed(fn):
        for _ in range(2):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    out = {}
    N, d, T, V = cfg.n_rollouts, cfg.d, lp_hidden.shape[0], lm_head.shape[0]
    # stochastic policy (App. A.4): 4096-entry labelled buffer, 128 bins, then one Bernoulli prune of the batch
    s_buf, label, s_batch, uniforms = W.policy_inputs(cfg, dev)
    pol = A.Policy(0.5, 0.5, 0.5, 0.05, 0.95, 1.0)
    c_pos, c_neg = A.arrol_histogram(s_buf, label, 128)
    q_lut, p_lut, _ = A.arrol_calibrate(c_pos, c_neg, pol)
    out["histogram"] = {"ms": timed(lambda: A.arrol_histogram(s_buf, label, 128)), "shape": "M=%d, B=128" % s_buf.numel()}
    out["calibrate"] = {"ms": timed(lambda: A.arrol_calibrate(c_pos, c_neg, pol)), "shape": "B=128, 64 bisection steps"}
    out["prune_bernoulli"] = {"ms": timed(lambda: A.arrol_prune_bernoulli(s_batch, uniforms, p_lut)),
                              "shape": "N=%d" % s_batch.numel()}
    # quality head variants on the batch's checkpoint hidden states
    hidden, w, bias, labels = W.head_training_inputs(cfg, dev)
    m = 512
    g = torch.Generator(device=dev); g.manual_seed(77)
    w1 = (torch.randn(m, d, generator=g, device=dev) * d ** -0.5).to(torch.bfloat16)
    b1 = torch.zeros(m, device=dev)
    w2 = torch.randn(m, generator=g, device=dev) * m ** -0.5
    ms = timed(lambda: A.arrol_score_mlp(hidden, w1, b1, w2))
    out["score_mlp"] = {"ms": ms, "shape": "N=%d, d=%d, m=%d" % (N, d, m), "TFLOPs": 2.0 * N * d * m / ms / 1e9}
    mws = torch.empty(max(256, A.lib().arrol_score_mlp_grad_workspace_bytes(N, d, m)), dtype=torch.uint8, device=dev)
    ms = timed(lambda: A.arrol_score_mlp_grad(hidden, w1, b1, w2, 0.0, labels, workspace=mws))
    out["score_mlp_grad"] = {"ms": ms, "shape": "N=%d, d=%d, m=%d" % (N, d, m), "TFLOPs": 6.0 * N * d * m / ms / 1e9}
    gws = torch.empty(max(16, A.lib().arrol_score_grad_workspace_bytes(N, d)), dtype=torch.uint8, device=dev)
    ms = timed(lambda: A.arrol_score_grad(hidden, w, bias, labels, workspace=gws))
    out["score_grad"] = {"ms": ms, "shape": "N=%d, d=%d" % (N, d), "GBps": N * d * 2 / ms / 1e6}
    _, gw, _ = A.arrol_score_grad(hidden, w, bias, labels, workspace=gws)
    wt, m1, v1 = w.clone(), torch.zeros_like(w), torch.zeros_like(w)
    out["adamw_step"] = {"ms": timed(lambda: A.arrol_adamw_step(wt, gw, m1, v1, 1, 1e-3)), "shape": "n=%d" % d}
    # trace confidence on the survivors' response tokens (lse from the log-prob pass)
    lp = torch.empty(T, dtype=torch.float32, device=dev)
    lse = torch.empty(T, dtype=torch.float32, device=dev)
    A.arrol_logprob(lp_hidden, lm_head, targets, out_logprob=lp, out_lse=lse, workspace=lws)
    cws = torch.empty(max(16, A.lib().arrol_token_confidence_workspace_bytes(V, d)), dtype=torch.uint8, device=dev)
    ms = timed(lambda: A.arrol_token_confidence(lp_hidden, lm_head, lse, workspace=cws))
    by = V * d * 2.0 + T * d * 2.0 + T * 8.0
    out["token_confidence"] = {"ms": ms, "shape": "T=%d, V=%d, d=%d" % (T, V, d), "GBps": by / ms / 1e6,
                               "frac_of_hbm_peak": by / ms / 1e6 / HBM_PEAK_GBPS}
    conf = A.arrol_token_confidence(lp_hidden, lm_head, lse, workspace=cws)
    cud = cu.to(dev)
    n_seq = cud.numel() - 1
    tws = torch.empty(max(16, A.lib().arrol_trace_confidence_workspace_bytes(T, n_seq)), dtype=torch.uint8, device=dev)
    out["trace_confidence"] = {"ms": timed(lambda: A.arrol_trace_confidence(conf, cud, 2048, 10, workspace=tws)),
                               "shape": "%d traces, T=%d, window 2048, bottom 10 %%" % (n_seq, T)}
    # GRPO advantage and objective on the survivors (reference log-probs = current ones plus noise)
    reward = (torch.rand(n_seq, generator=g, device=dev) < 0.5).to(torch.float32)
    off = torch.arange(0, n_seq + 1, cfg.K, dtype=torch.int64, device=dev)
    lp_ref = lp + 0.2 * torch.randn(T, generator=g, device=dev)
    out["grpo_advantage"] = {"ms": timed(lambda: A.arrol_grpo_advantage(reward, off)),
                             "shape": "%d groups of %d" % (off.numel() - 1, cfg.K)}
    adv, wgt = A.arrol_grpo_advantage(reward, off)
    ows = torch.empty(max(16, A.lib().arrol_grpo_objective_workspace_bytes(n_seq)), dtype=torch.uint8, device=dev)
    out["grpo_objective"] = {"ms": timed(lambda: A.arrol_grpo_objective(lp, lp_ref, cud, adv, wgt, 0.2, 0.2, 0.01,
                                                                        workspace=ows)),
                             "shape": "T=%d, %d rollouts, with gradient" % (T, n_seq)}
    for v in out.values():
        for k in list(v):
            if isinstance(v[k], float):
                v[k] = round(v[k], 5)
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported. "
              "Data parallelism over prompt groups needs no exchange: run one process per GPU." % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the ARRoL path has no CPU implementation", file=sys.stderr)
        sys.exit(2)
    if args.calibrate_copy:
        calibrate_copy(torch)
        return
    import paper_2603_24840_amd as A
    from paper_2603_24840_amd import workloads as W

    A.lib()
    for kv in (x for x in args.tune.split(",") if x):
        k, v = kv.split("=")
        A.set_tuning(k, int(v))
    dev = "cuda:0"
    cfg = W.CONFIGS[args.workload]
    only = set(x for x in args.only.split(",") if x)
    run = lambda s: not only or s in only

    # ---- inputs, resident in HBM before anything is timed ------------------------------------
    hidden, w, bias = W.score_inputs(cfg, dev)
    kv_src, block_table, seq_len, tokens = W.compact_inputs(cfg, dev)
    lp_hidden, lm_head, targets, cu = W.logprob_inputs(cfg, dev)
    vote_hidden, answer_id = W.vote_inputs(cfg, dev)
    T = lp_hidden.shape[0]
    N, Nk, ppr = cfg.n_rollouts, cfg.n_keep, cfg.pages_per_rollout
    n_vote = cfg.vote_q * cfg.vote_c
    # the vote runs on the batch's own probabilities when Q*C fits in it (one question per prompt
    # group); a larger test-time shape scores its own candidates inside the vote stage
    vote_own_score = n_vote > N
    vote_prob = torch.empty(n_vote, dtype=torch.float32, device=dev) if vote_own_score else None
    if not vote_own_score:
        del vote_hidden

    # ---- outputs and workspaces, allocated once -----------------------------------------------
    score_o = torch.empty(N, dtype=torch.float32, device=dev)
    prob = torch.empty(N, dtype=torch.float32, device=dev)
    keep = torch.empty(N, dtype=torch.uint8, device=dev)
    surv = torch.empty(Nk, dtype=torch.int32, device=dev)
    kv_dst = torch.empty((cfg.n_layers, 2, Nk * ppr) + tuple(kv_src.shape[3:]), dtype=torch.bfloat16, device=dev)
    cout = dict(block_table_dst=torch.empty((Nk, ppr), dtype=torch.int32, device=dev),
                seq_len_dst=torch.empty(Nk, dtype=torch.int32, device=dev),
                tokens_dst=torch.empty((Nk, tokens.shape[1]), dtype=torch.int32, device=dev),
                src_of_dst=torch.empty(Nk, dtype=torch.int32, device=dev),
                n_pages_used=torch.empty(1, dtype=torch.int64, device=dev))
    cws = torch.empty(max(16, A.arrol_compact_workspace_bytes(Nk)), dtype=torch.uint8, device=dev)
    logprob = torch.empty(T, dtype=torch.float32, device=dev)
    lws = torch.empty(max(16, A.arrol_logprob_workspace_bytes(T, cfg.vocab, cfg.d)), dtype=torch.uint8, device=dev)

    stages = ["score", "select", "compact", "logprob", "vote"]
    stage_ms = {s: 0.0 for s in stages}

    def step(events=None):
        def mark(i):
            if events is not None:
                events[i].record()
        mark(0)
        if run("score"):
            A.arrol_score(hidden, w, bias, out_score=score_o, out_prob=prob)
        mark(1)
        if run("select"):
            A.arrol_select(prob, cfg.n_prompts, cfg.G, cfg.K, cfg.rho, out_keep=keep, out_survivors=surv)
        mark(2)
        if run("compact"):
            A.arrol_compact(kv_src, kv_dst, block_table, seq_len, tokens, surv, out=cout, workspace=cws)
        mark(3)
        if run("logprob"):
            A.arrol_logprob(lp_hidden, lm_head, targets, out_logprob=logprob, workspace=lws)
        mark(4)
        if run("vote"):
            if vote_own_score:
                A.arrol_score(vote_hidden, w, bias, want_score=False, out_prob=vote_prob)
                A.arrol_weighted_vote(vote_prob, answer_id, cfg.vote_q, cfg.vote_c, cfg.vote_a)
            else:
                A.arrol_weighted_vote(prob[:n_vote], answer_id, cfg.vote_q, cfg.vote_c, cfg.vote_a)
        mark(5)

    if only and "select" not in only:   # a profiling run that skips selection still needs survivors
        A.arrol_score(hidden, w, bias, out_score=score_o, out_prob=prob)
        A.arrol_select(prob, cfg.n_prompts, cfg.G, cfg.K, cfg.rho, out_keep=keep, out_survivors=surv)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(evs[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    for k in range(args.steps):
        for i, s in enumerate(stages):
            stage_ms[s] += evs[k][i].elapsed_time(evs[k][i + 1]) / args.steps
    ms_per_step = wall * 1e3 / args.steps

    # ---- algorithmic work ----------------------------------------------------------------------
    flop = 2.0 * T * cfg.vocab * cfg.d
    kv_bytes = 2.0 * cfg.n_layers * 2 * Nk * ppr * cfg.chunk_bytes        # survivor KV read once + written once
    meta_bytes = 2.0 * Nk * (ppr + tokens.shape[1] + 2) * 4
    prune_bytes = N * cfg.d * 2 + cfg.d * 4 + N * 8 + N * 4 + N + 4 * Nk
    lp_s = stage_ms["logprob"] / 1e3
    cp_s = stage_ms["compact"] / 1e3
    achieved_tflops = flop / lp_s / 1e12 if lp_s > 0 else 0.0
    pc_s = (stage_ms["score"] + stage_ms["select"] + stage_ms["compact"]) / 1e3
    result = {
        "metric": "log-prob tokens/s over the whole prune+compact+log-prob step (1 GPU)",
        "value": T / (ms_per_step / 1e3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %d prompts x G=%d keep K=%d, d=%d, checkpoint %d tokens, KV %dL x %dH x %d "
                               "page %d, vocab %d, T=%d response tokens (lengths U[%d,%d]); vote %dx%d over %d answers"
                               % (cfg.name, cfg.n_prompts, cfg.G, cfg.K, cfg.d, cfg.ckpt_len, cfg.n_layers,
                                  cfg.n_kv_heads, cfg.head_dim, cfg.page_tokens, cfg.vocab, T, cfg.resp_lo,
                                  cfg.resp_hi, cfg.vote_q, cfg.vote_c, cfg.vote_a),
                   "stages_run": sorted(only) if only else stages},
        "roofline": {"bound": "mfma", "kernel": "logprob_kernel (+ split merge)",
                     "achieved": achieved_tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved_tflops / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": PROFILED_TRAFFIC_BYTES.get((cfg.name, "logprob"))},
        "roofline_compact": {"bound": "hbm", "kernel": "compact_copy_kernel (+ plan)",
                             "achieved": (kv_bytes + meta_bytes) / cp_s / 1e9 if cp_s > 0 else 0.0,
                             "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                             "frac": (kv_bytes + meta_bytes) / cp_s / 1e9 / HBM_PEAK_GBPS if cp_s > 0 else 0.0,
                             "traffic": PROFILED_TRAFFIC_BYTES.get((cfg.name, "compact"))},
        "prune_compact_GBps": (prune_bytes + kv_bytes + meta_bytes) / pc_s / 1e9 if pc_s > 0 else 0.0,
        # algorithmic bytes of each HBM-bound stage over its own event time (score and select are
        # launch-latency bound at training shapes: a few microseconds for a few megabytes)
        "stage_GBps": {"score": (N * cfg.d * 2 + cfg.d * 4 + N * 8) / stage_ms["score"] / 1e6 if stage_ms["score"] > 0 else 0.0,
                       "select": (N * 4 + N + 4 * Nk) / stage_ms["select"] / 1e6 if stage_ms["select"] > 0 else 0.0,
                       "compact": (kv_bytes + meta_bytes) / stage_ms["compact"] / 1e6 if stage_ms["compact"] > 0 else 0.0},
        "logprob_tokens_per_s": T / lp_s if lp_s > 0 else 0.0,
        "stage_ms": {k: round(v, 4) for k, v in stage_ms.items()},
        "paper_context": "the paper reports no kernel-level number for this path; its end-to-end RLVR training "
                         "speedup is 1.6-1.7x (up to 1.7x) on NVIDIA GH200 GPUs: other hardware, another metric, "
                         "context only",
    }
    if args.inplace_compaction:
        # the in-place variant rewrites the pool, so the pool is restored (untimed) before every call
        orig = kv_src.clone()
        iws = torch.empty(max(16, A.lib().arrol_compact_inplace_workspace_bytes(kv_src.shape[2])), dtype=torch.uint8, device=dev)
        times = []
        for _ in range(args.warmup + args.steps):
            kv_src.copy_(orig)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            iout = A.arrol_compact_inplace(kv_src, block_table, seq_len, surv, workspace=iws)
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
        kv_src.copy_(orig)
        del orig
        ms = sum(times[args.warmup:]) / args.steps
        moved = int(iout["n_moved"][0])
        moved_bytes = 2.0 * moved * cfg.n_layers * 2 * cfg.chunk_bytes
        result["compact_inplace"] = {"ms": ms, "pages_live": int(iout["n_pages_used"][0]), "pages_moved": moved,
                                     "bytes_read_plus_written": moved_bytes, "GBps": moved_bytes / ms / 1e6,
                                     "frac_of_hbm_peak": moved_bytes / ms / 1e6 / HBM_PEAK_GBPS}
    if not only:
        result["roofline_score"] = time_score_test_time_shape(A, W, dev, torch)
    if args.extras:
        result["extras"] = time_extras(A, W, cfg, dev, torch, lp_hidden, lm_head, targets, cu, lws)
    if not args.skip_cpu_baseline and not only:
        tensors = dict(hidden=hidden, w=w, bias=bias, surv=surv, kv_src=kv_src, kv_dst=kv_dst,
                       block_table=block_table, seq_len=seq_len, tokens=tokens, lp_hidden=lp_hidden,
                       lm_head=lm_head, targets=targets, logprob=logprob, answer_id=answer_id,
                       vote_hidden=vote_hidden if vote_own_score else None)
        result["cpu_baseline"] = cpu_baseline(cfg, tensors, args.cpu_sample_rows, torch)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
