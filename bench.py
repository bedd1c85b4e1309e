"""Benchmark of the ARRoL pruning path on one MI355X.

A step is one pass of the whole hot path over one synthetic batch:
  arrol_score -> arrol_select -> arrol_compact -> arrol_logprob -> arrol_weighted_vote
all enqueued on one stream with no host synchronisation in between.  Inputs are resident in
HBM before the timed region.  Prints ONE JSON line.

The headline workload is the largest configuration (qwen8b: Qwen3-8B-shaped, 155 GB KV pool,
2.36 M response tokens); the other four configurations are then run for a few steps each and
reported, with their own rooflines and oracle parity on a sample, under "all_configs".

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload qwen8b] [--skip-cpu-baseline]
                  [--skip-all-configs]
  python bench.py --calibrate-copy      # plain 1 GiB device copy, for scaling rocprof byte counters
  python bench.py --extras              # adds timings of the calls outside the five-stage step
  python bench.py --only logprob --input-data zeros   # profiling aids (see profiles/)
  python bench.py --only logprob --mfma-probe         # register-only MFMA rate of this card beside the kernel's
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak, published
STAGES = ["score", "select", "compact", "logprob", "vote"]
ALL_WORKLOADS = ["tiny", "llama1b", "qwen1p7b", "llama3b", "qwen8b"]

# HBM-side bytes per launch of the two dominant kernels, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs of this file scaled by the plain-copy calibration; one summary per workload under profiles/
# (hbm_traffic_<workload>.txt).  For the log-prob kernel the figure is the fetch at the L2 <-> fabric
# interface, Infinity-Cache hits included.  None where not measured.
PROFILED_TRAFFIC_BYTES = {
    ("llama1b", "logprob"): 3.3619e+11, ("llama1b", "compact"): 8.5949e+09,
    ("qwen1p7b", "logprob"): 1.0884e+12, ("qwen1p7b", "compact"): 1.2027e+11,
    ("llama3b", "logprob"): 1.7869e+12, ("llama3b", "compact"): 1.2027e+11,
    ("qwen8b", "logprob"): 4.4537e+12, ("qwen8b", "compact"): 1.5464e+11,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="qwen8b", choices=ALL_WORKLOADS)
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--skip-all-configs", action="store_true",
                    help="do not run the other four configurations after the headline workload")
    ap.add_argument("--cpu-sample-rows", type=int, default=1536,
                    help="log-prob rows the oracle computes for cpu_baseline (edge rows always included)")
    ap.add_argument("--config-steps", type=int, default=3, help="timed steps per entry of all_configs")
    ap.add_argument("--config-sample-rows", type=int, default=128,
                    help="log-prob rows the oracle checks per entry of all_configs")
    ap.add_argument("--calibrate-copy", action="store_true")
    ap.add_argument("--inplace-compaction", action="store_true",
                    help="also time arrol_compact_inplace on the same pool and survivors (extra JSON object)")
    ap.add_argument("--extras", action="store_true",
                    help="also time the entry points outside the five-stage step (stochastic policy, MLP head, head "
                         "training, trace confidence, GRPO objective) on the same workload (extra JSON object)")
    ap.add_argument("--logprob-splits", type=int, default=0, help="n_splits passed to arrol_logprob (0 = library's choice)")
    ap.add_argument("--input-data", default="randn", choices=["randn", "zeros"],
                    help="contents of the log-prob operands: the workload's N(0,1) recipe, or all zeros "
                         "(same kernel and launch, no operand toggling: shows the clock the part reaches without a power limit)")
    ap.add_argument("--mfma-probe", action="store_true",
                    help="also with --only / --input-data: time the register-only MFMA loops (on by default otherwise)")
    ap.add_argument("--skip-mfma-probe", action="store_true")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="also time the ROCm BLAS bf16 GEMM (torch.matmul) on the first 32,768 rows of the same log-prob "
                         "operands: the matrix throughput a vendor-tuned kernel sustains on this data, for context")
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


def host_threads():
    """(logical CPUs of this machine, threads the oracle's BLAS calls really use)."""
    n_cpu = os.cpu_count()
    try:
        from threadpoolctl import threadpool_info
        blas = [p.get("num_threads", 0) for p in threadpool_info() if p.get("user_api") == "blas"]
        return n_cpu, (max(blas) if blas else 1)
    except Exception:
        return n_cpu, None


def describe(cfg, T):
    return ("%s: %d prompts x G=%d keep K=%d, d=%d, checkpoint %d tokens, KV %dL x %dH x %d page %d, vocab %d, "
            "T=%d response tokens (lengths U[%d,%d]); vote %dx%d over %d answers"
            % (cfg.name, cfg.n_prompts, cfg.G, cfg.K, cfg.d, cfg.ckpt_len, cfg.n_layers, cfg.n_kv_heads, cfg.head_dim,
               cfg.page_tokens, cfg.vocab, T, cfg.resp_lo, cfg.resp_hi, cfg.vote_q, cfg.vote_c, cfg.vote_a))


class Workload:
    """Inputs, outputs and workspaces of one configuration, all resident in HBM."""

    def __init__(self, A, W, torch, cfg, dev, input_data="randn", n_splits=0):
        self.A, self.W, self.torch, self.cfg, self.dev = A, W, torch, cfg, dev
        self.n_splits = n_splits
        self.hidden, self.w, self.bias = W.score_inputs(cfg, dev)
        self.kv_src, self.block_table, self.seq_len, self.tokens = W.compact_inputs(cfg, dev)
        self.lp_hidden, self.lm_head, self.targets, self.cu = W.logprob_inputs(cfg, dev)
        if input_data == "zeros":
            self.lp_hidden.zero_()
            self.lm_head.zero_()
        self.vote_hidden, self.answer_id = W.vote_inputs(cfg, dev)
        self.T = self.lp_hidden.shape[0]
        N, Nk, ppr = cfg.n_rollouts, cfg.n_keep, cfg.pages_per_rollout
        self.n_vote = cfg.vote_q * cfg.vote_c
        # the vote runs on the batch's own probabilities when Q*C fits in it (one question per prompt
        # group); a larger test-time shape scores its own candidates inside the vote stage
        self.vote_own_score = self.n_vote > N
        self.vote_prob = torch.empty(self.n_vote, dtype=torch.float32, device=dev) if self.vote_own_score else None
        if not self.vote_own_score:
            self.vote_hidden = None
        f32 = lambda *shape: torch.empty(shape, dtype=torch.float32, device=dev)
        i32 = lambda *shape: torch.empty(shape, dtype=torch.int32, device=dev)
        self.score_o, self.prob = f32(N), f32(N)
        self.keep = torch.empty(N, dtype=torch.uint8, device=dev)
        self.surv = i32(Nk)
        self.kv_dst = torch.empty((cfg.n_layers, 2, Nk * ppr) + tuple(self.kv_src.shape[3:]), dtype=torch.bfloat16,
                                  device=dev)
        self.cout = dict(block_table_dst=i32(Nk, ppr), seq_len_dst=i32(Nk), tokens_dst=i32(Nk, self.tokens.shape[1]),
                         src_of_dst=i32(Nk), n_pages_used=torch.empty(1, dtype=torch.int64, device=dev))
        self.cws = torch.empty(max(16, A.arrol_compact_workspace_bytes(Nk)), dtype=torch.uint8, device=dev)
        self.logprob = f32(self.T)
        self.lws = torch.empty(max(16, A.arrol_logprob_workspace_bytes(self.T, cfg.vocab, cfg.d, n_splits)),
                               dtype=torch.uint8, device=dev)
        self.winner = i32(cfg.vote_q)

    def step(self, run, events=None):
        A, cfg = self.A, self.cfg

        def mark(i):
            if events is not None:
                events[i].record()
        mark(0)
        if run("score"):
            A.arrol_score(self.hidden, self.w, self.bias, out_score=self.score_o, out_prob=self.prob)
        mark(1)
        if run("select"):
            A.arrol_select(self.prob, cfg.n_prompts, cfg.G, cfg.K, cfg.rho, out_keep=self.keep, out_survivors=self.surv)
        mark(2)
        if run("compact"):
            A.arrol_compact(self.kv_src, self.kv_dst, self.block_table, self.seq_len, self.tokens, self.surv,
                            out=self.cout, workspace=self.cws)
        mark(3)
        if run("logprob"):
            A.arrol_logprob(self.lp_hidden, self.lm_head, self.targets, out_logprob=self.logprob,
                            n_splits=self.n_splits, workspace=self.lws)
        mark(4)
        if run("vote"):
            if self.vote_own_score:
                A.arrol_score(self.vote_hidden, self.w, self.bias, want_score=False, out_prob=self.vote_prob)
                A.arrol_weighted_vote(self.vote_prob, self.answer_id, cfg.vote_q, cfg.vote_c, cfg.vote_a,
                                      out_winner=self.winner)
            else:
                A.arrol_weighted_vote(self.prob[:self.n_vote], self.answer_id, cfg.vote_q, cfg.vote_c, cfg.vote_a,
                                      out_winner=self.winner)
        mark(5)

    def time_steps(self, steps, warmup, only=()):
        """W untimed steps, then K timed ones bracketed by synchronisation; per-stage times from HIP events
        recorded on the stream the kernels are launched on (torch's current stream)."""
        torch = self.torch
        run = lambda s: not only or s in only
        if only and "select" not in only:   # a profiling run that skips selection still needs survivors
            self.A.arrol_score(self.hidden, self.w, self.bias, out_score=self.score_o, out_prob=self.prob)
            self.A.arrol_select(self.prob, self.cfg.n_prompts, self.cfg.G, self.cfg.K, self.cfg.rho,
                                out_keep=self.keep, out_survivors=self.surv)
        for _ in range(warmup):
            self.step(run)
        torch.cuda.synchronize()
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(steps)]
        t0 = time.perf_counter()
        for k in range(steps):
            self.step(run, evs[k])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        stage_ms = {s: (sum(evs[k][i].elapsed_time(evs[k][i + 1]) for k in range(steps)) / steps if run(s) else None)
                    for i, s in enumerate(STAGES)}
        return wall * 1e3 / steps, stage_ms

    def work(self):
        """Algorithmic work per step: log-prob FLOP, compaction bytes (survivor KV read once + written once,
        plus the metadata), bytes of the prune stages."""
        cfg, Nk, ppr, N = self.cfg, self.cfg.n_keep, self.cfg.pages_per_rollout, self.cfg.n_rollouts
        flop = 2.0 * self.T * cfg.vocab * cfg.d
        kv_bytes = 2.0 * cfg.n_layers * 2 * Nk * ppr * cfg.chunk_bytes
        meta_bytes = 2.0 * Nk * (ppr + self.tokens.shape[1] + 2) * 4
        score_bytes = N * cfg.d * 2 + cfg.d * 4 + N * 8
        select_bytes = N * 4 + N + 4 * Nk
        return flop, kv_bytes + meta_bytes, score_bytes, select_bytes

    def report(self, ms_per_step, stage_ms):
        """Rooflines of the two dominant kernels and the per-stage rates.  A stage that did not run yields null
        figures (never a rate computed from a missing time)."""
        cfg = self.cfg
        flop, compact_bytes, score_bytes, select_bytes = self.work()
        rate = lambda amount, ms, scale: (amount / ms / scale) if ms else None
        tflops = rate(flop, stage_ms["logprob"], 1e9)
        c_gbps = rate(compact_bytes, stage_ms["compact"], 1e6)
        pc = [stage_ms[s] for s in ("score", "select", "compact")]
        frac = lambda x, peak: (x / peak) if x is not None else None
        return {
            "roofline": {"bound": "mfma",
                         "kernel": "logprob_ring_kernel (+ logprob_finalize_kernel, the split merge)" if cfg.d % 64 == 0
                                   else "logprob_kernel (+ logprob_finalize_kernel)",
                         "achieved": tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": frac(tflops, MFMA_BF16_PEAK_TFLOPS),
                         "traffic": PROFILED_TRAFFIC_BYTES.get((cfg.name, "logprob"))},
            "roofline_compact": {"bound": "hbm", "kernel": "compact_copy_kernel (+ compact_plan_kernel)",
                                 "achieved": c_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                 "frac": frac(c_gbps, HBM_PEAK_GBPS),
                                 "traffic": PROFILED_TRAFFIC_BYTES.get((cfg.name, "compact"))},
            "prune_compact_GBps": rate(score_bytes + select_bytes + compact_bytes, sum(pc), 1e6) if all(pc) else None,
            # algorithmic bytes of each HBM-side stage over its own event time (score and select are
            # launch-latency bound at training shapes: a few microseconds for a few megabytes)
            "stage_GBps": {"score": rate(score_bytes, stage_ms["score"], 1e6),
                           "select": rate(select_bytes, stage_ms["select"], 1e6), "compact": c_gbps},
            "logprob_tokens_per_s": rate(self.T, stage_ms["logprob"], 1e-3),
            "stage_ms": {k: (round(v, 4) if v is not None else None) for k, v in stage_ms.items()},
        }

    def oracle_check(self, sample_rows, timed=False):
        """The oracle's own chain from the seeded inputs (never from a library output), on a bounded sample of
        this step: score / select / vote on the full batch, compaction on the first and the last KV layer,
        log-prob on `sample_rows` seeded rows plus the mandatory edge rows.  Returns (stage seconds scaled to the
        full step, parity figures, description of the sample)."""
        import numpy as np
        import oracle as O
        W, cfg, torch = self.W, self.cfg, self.torch
        bits, npy = W.bits, W.npy
        times = {}
        t0 = time.perf_counter()
        _, q = O.score(bits(self.hidden), npy(self.w), self.bias)
        times["score"] = time.perf_counter() - t0
        score_err = float(np.max(np.abs(npy(self.prob).astype(np.float64) - q)))
        q32 = q.astype(np.float32)            # the oracle's own chain: its probabilities at the interface precision
        t0 = time.perf_counter()
        _, surv = O.select(q32, cfg.n_prompts, cfg.G, cfg.K, cfg.rho)
        times["select"] = time.perf_counter() - t0
        select_ok = bool(np.array_equal(npy(self.surv), surv))
        # compact: the first and the last layer of the pool (lowest and highest addresses); layers are
        # independent slabs, so the host time is scaled by layers / sampled layers
        layers = sorted({0, cfg.n_layers - 1})
        bt, sl, tok = npy(self.block_table), npy(self.seq_len), npy(self.tokens)
        compact_ok, host_s = True, 0.0
        for layer in layers:
            kv_host = bits(self.kv_src[layer:layer + 1])
            t0 = time.perf_counter()
            ref = O.compact(kv_host, bt, sl, tok, surv, self.kv_dst.shape[2])
            host_s += time.perf_counter() - t0
            compact_ok = compact_ok and bool(np.array_equal(bits(self.kv_dst[layer:layer + 1]), ref["kv_dst"]))
            del kv_host
        times["compact"] = host_s * cfg.n_layers / len(layers)
        for k in ("block_table_dst", "seq_len_dst", "tokens_dst", "src_of_dst"):
            compact_ok = compact_ok and bool(np.array_equal(npy(self.cout[k]), ref[k]))
        compact_ok = compact_ok and int(self.cout["n_pages_used"][0]) == ref["n_pages_used"]
        del ref
        # logprob: seeded rows plus row 0, row T-1, first / last row of the first / last survivor, and the rows
        # whose targets are 0, V-1 and on the first and last vocabulary-tile edge
        rows = W.logprob_check_rows(self.T, sample_rows, cfg.vocab, self.cu)
        h_s = bits(self.lp_hidden[rows.to(self.dev)])
        w_b = bits(self.lm_head)
        y_s = npy(self.targets)[rows.numpy()]
        t0 = time.perf_counter()
        lp_o, _ = O.logprob(h_s, w_b, y_s)
        times["logprob"] = (time.perf_counter() - t0) * self.T / len(rows)
        lp_err = float(np.max(np.abs(npy(self.logprob)[rows.numpy()].astype(np.float64) - lp_o)))
        del w_b, h_s
        t0 = time.perf_counter()
        if self.vote_own_score:               # test-time shape: the vote stage scored its own candidates
            vote_q32 = O.score(bits(self.vote_hidden), npy(self.w), self.bias)[1].astype(np.float32)
        else:                                 # the vote ran on the batch's own probabilities
            vote_q32 = q32[:self.n_vote]
        win_o, _ = O.weighted_vote(vote_q32, npy(self.answer_id), cfg.vote_q, cfg.vote_c, cfg.vote_a)
        times["vote"] = time.perf_counter() - t0
        vote_ok = bool(np.array_equal(npy(self.winner), win_o))
        parity = {"prob_max_abs_err": score_err, "select_identical": select_ok, "compact_bit_exact": compact_ok,
                  "compact_layers_checked": layers, "logprob_max_abs_err": lp_err, "logprob_rows_checked": len(rows),
                  "vote_identical": vote_ok,
                  "ok": bool(score_err < 1e-3 and select_ok and compact_ok and lp_err < 2e-3 and vote_ok)}
        sample = ("score/select/vote on the full batch; compact on layers %s of %d; logprob on %d of %d rows (seeded, "
                  "incl. row 0, row T-1, first/last row of the first/last survivor, targets 0, V-1 and on vocabulary-tile "
                  "edges); stage times scaled to the full step" % (layers, cfg.n_layers, len(rows), self.T))
        return times, parity, sample


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


def time_vendor_gemm(wl, torch, rows=32768, reps=10):
    """torch.matmul (the ROCm BLAS bf16 GEMM, logits written to memory) on the first `rows` rows of the same
    log-prob operands.  Not part of the path: it shows what a vendor-tuned plain GEMM sustains on this data."""
    n = min(rows, wl.T)
    H, Wt = wl.lp_hidden[:n], wl.lm_head.t()
    out = torch.empty((n, wl.cfg.vocab), dtype=torch.bfloat16, device=wl.dev)
    for _ in range(reps):
        torch.matmul(H, Wt, out=out)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        torch.matmul(H, Wt, out=out)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    tf = 2.0 * n * wl.cfg.vocab * wl.cfg.d / ms / 1e9
    del out
    return {"what": "torch.matmul bf16 [%d x %d] x [%d x %d]^T, logits stored; library GEMM, not this path"
                    % (n, wl.cfg.d, wl.cfg.vocab, wl.cfg.d), "ms": ms, "TFLOPs": tf, "frac_of_peak": tf / MFMA_BF16_PEAK_TFLOPS}


def time_mfma_probe(A, wl, torch, iters=300000):
    """Register-only bf16 MFMA loops (arrol_probe_mfma_rate: no LDS, no memory traffic, 2 wavefronts per SIMD on all
    256 CUs) on the first values of the log-prob operands and on zeros: what this card's matrix cores sustain under
    its power limit.  Not part of the path; it puts the log-prob kernel's rate beside the card's own ceiling."""
    n = min(64 * 8 * 12 * 256, wl.lp_hidden.numel() // 512 * 512, wl.lm_head.numel() // 512 * 512)
    a_r, b_r = wl.lp_hidden.reshape(-1)[:n].contiguous(), wl.lm_head.reshape(-1)[:n].contiguous()
    zeros = torch.zeros(n, dtype=torch.bfloat16, device=wl.dev)
    sink = torch.empty(256 * 512, dtype=torch.float32, device=wl.dev)
    out = {"what": "v_mfma bf16 from registers only, 256 workgroups x 8 wavefronts, %d iterations of 32 (16) "
                   "instructions per wavefront; TFLOP/s by HIP events" % iters}
    for data, (a, b) in (("randn", (a_r, b_r)), ("zeros", (zeros, zeros))):
        out[data] = {}
        for shape, name in ((16, "16x16x32"), (32, "32x32x16")):
            A.arrol_probe_mfma_rate(a, b, shape=shape, iters=iters // 3, out_sink=sink)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            _, flop = A.arrol_probe_mfma_rate(a, b, shape=shape, iters=iters, out_sink=sink)
            e1.record()
            torch.cuda.synchronize()
            out[data][name] = round(flop / e0.elapsed_time(e1) / 1e9, 1)
    out["frac_of_peak_randn_16x16x32"] = out["randn"]["16x16x32"] / MFMA_BF16_PEAK_TFLOPS
    return out


def time_extras(A, W, cfg, dev, torch, lp_hidden, lm_head, targets, cu, reps=10):
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
    sws_bytes = A.lib().arrol_score_mlp_workspace_bytes(N, d, m)
    sws = torch.empty(sws_bytes, dtype=torch.uint8, device=dev) if sws_bytes else None
    ms = timed(lambda: A.arrol_score_mlp(hidden, w1, b1, w2, workspace=sws))
    out["score_mlp"] = {"ms": ms, "shape": "N=%d, d=%d, m=%d" % (N, d, m), "TFLOPs": 2.0 * N * d * m / ms / 1e9,
                        "path": "small-batch (wavefront per 32x32 block + finish)" if sws_bytes else "tile kernel",
                        "note": "HIP-event mean over back-to-back calls from Python: a floor of ~20 us per call is host launch cost; "
                                "kernel durations are in profiles/"}
    mws = torch.empty(max(256, A.lib().arrol_score_mlp_grad_workspace_bytes(N, d, m, 1)), dtype=torch.uint8, device=dev)
    ms = timed(lambda: A.arrol_score_mlp_grad(hidden, w1, b1, w2, 0.0, labels, workspace=mws))
    out["score_mlp_grad"] = {"ms": ms, "shape": "N=%d, d=%d, m=%d" % (N, d, m), "TFLOPs": 4.0 * N * d * m / ms / 1e9,
                             "flops": "two contractions (forward, dL/dW1): 4*N*d*m; the pre-activations are kept, not recomputed"}
    # the MLP head at the test-time-scaling shape of the largest configuration
    big = W.CONFIGS["qwen8b"]
    nb = big.vote_q * big.vote_c
    hb = W.randn_bf16((nb, big.d), g, dev)
    w1b = (torch.randn(m, big.d, generator=g, device=dev) * big.d ** -0.5).to(torch.bfloat16)
    lb = (torch.rand(nb, generator=g, device=dev) < 0.5).to(torch.float32)
    ms = timed(lambda: A.arrol_score_mlp(hb, w1b, b1, w2))
    out["score_mlp_test_time_shape"] = {"ms": ms, "shape": "N=%d, d=%d, m=%d" % (nb, big.d, m),
                                        "TFLOPs": 2.0 * nb * big.d * m / ms / 1e9}
    bws = torch.empty(max(256, A.lib().arrol_score_mlp_grad_workspace_bytes(nb, big.d, m, 1)), dtype=torch.uint8, device=dev)
    ms = timed(lambda: A.arrol_score_mlp_grad(hb, w1b, b1, w2, 0.0, lb, workspace=bws))
    out["score_mlp_grad_test_time_shape"] = {"ms": ms, "shape": "N=%d, d=%d, m=%d" % (nb, big.d, m),
                                             "TFLOPs": 4.0 * nb * big.d * m / ms / 1e9,
                                             "flops": "two contractions (forward, dL/dW1): 4*N*d*m"}
    del hb, w1b, lb, bws
    gws = torch.empty(max(16, A.lib().arrol_score_grad_workspace_bytes(N, d)), dtype=torch.uint8, device=dev)
    ms = timed(lambda: A.arrol_score_grad(hidden, w, bias, labels, workspace=gws))
    out["score_grad"] = {"ms": ms, "shape": "N=%d, d=%d" % (N, d), "GBps": N * d * 2 / ms / 1e6}
    _, gw, _ = A.arrol_score_grad(hidden, w, bias, labels, workspace=gws)
    wt, m1, v1 = w.clone(), torch.zeros_like(w), torch.zeros_like(w)
    out["adamw_step"] = {"ms": timed(lambda: A.arrol_adamw_step(wt, gw, m1, v1, 1, 1e-3)), "shape": "n=%d" % d}
    # trace confidence on the survivors' response tokens (lse from the log-prob pass)
    lp = torch.empty(T, dtype=torch.float32, device=dev)
    lse = torch.empty(T, dtype=torch.float32, device=dev)
    A.arrol_logprob(lp_hidden, lm_head, targets, out_logprob=lp, out_lse=lse)
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


def time_inplace(wl, torch, A, steps, warmup):
    """arrol_compact_inplace on the same pool and survivors.  The call copies live pages from above the live
    count onto dead pages below it and leaves every survivor's original pages intact, so repeating it with the
    same (original) block tables moves the same pages again: the pool needs no restoring between timed calls."""
    cfg, dev = wl.cfg, wl.dev
    iws = torch.empty(max(16, A.lib().arrol_compact_inplace_workspace_bytes(wl.kv_src.shape[2])), dtype=torch.uint8,
                      device=dev)
    times, iout = [], None
    for _ in range(warmup + steps):
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        iout = A.arrol_compact_inplace(wl.kv_src, wl.block_table, wl.seq_len, wl.surv, workspace=iws)
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1))
    ms = sum(times[warmup:]) / steps
    moved = int(iout["n_moved"][0])
    moved_bytes = 2.0 * moved * cfg.n_layers * 2 * cfg.chunk_bytes
    return {"ms": ms, "pages_live": int(iout["n_pages_used"][0]), "pages_moved": moved,
            "bytes_read_plus_written": moved_bytes, "GBps": moved_bytes / ms / 1e6,
            "frac_of_hbm_peak": moved_bytes / ms / 1e6 / HBM_PEAK_GBPS}


def run_config(A, W, torch, name, dev, steps, warmup, sample_rows):
    """One entry of all_configs: a few timed steps of the whole path plus oracle parity on a sample."""
    wl = Workload(A, W, torch, W.CONFIGS[name], dev)
    ms_per_step, stage_ms = wl.time_steps(steps, warmup)
    rep = wl.report(ms_per_step, stage_ms)
    _, parity, _ = wl.oracle_check(sample_rows)
    entry = {"workload": describe(wl.cfg, wl.T), "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
             "tokens_per_s": wl.T / (ms_per_step / 1e3),
             "logprob_frac_of_mfma_peak": rep["roofline"]["frac"], "logprob_TFLOPs": rep["roofline"]["achieved"],
             "logprob_traffic": rep["roofline"]["traffic"],
             "compact_frac_of_hbm_peak": rep["roofline_compact"]["frac"], "compact_GBps": rep["roofline_compact"]["achieved"],
             "stage_ms": rep["stage_ms"], "parity_on_sample": parity}
    del wl
    torch.cuda.empty_cache()
    return entry


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
    dev = "cuda:0"
    cfg = W.CONFIGS[args.workload]
    only = tuple(x for x in args.only.split(",") if x)
    profiling = bool(only) or args.input_data != "randn"

    # ---- inputs, resident in HBM before anything is timed ------------------------------------
    wl = Workload(A, W, torch, cfg, dev, input_data=args.input_data, n_splits=args.logprob_splits)
    ms_per_step, stage_ms = wl.time_steps(args.steps, args.warmup, only)
    result = {
        "metric": "log-prob tokens/s over the whole prune+compact+log-prob step (1 GPU)",
        "value": wl.T / (ms_per_step / 1e3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic" if args.input_data == "randn" else "synthetic (log-prob operands all zero)",
        "config": {"workload": describe(cfg, wl.T), "stages_run": list(only) if only else STAGES,
                   "logprob_n_splits": args.logprob_splits},
    }
    result.update(wl.report(ms_per_step, stage_ms))
    result["paper_context"] = ("the paper reports no kernel-level number for this path; its end-to-end RLVR training "
                               "speedup is 1.6-1.7x (up to 1.7x) on NVIDIA GH200 GPUs: other hardware, another metric, "
                               "context only")
    if args.inplace_compaction:
        result["compact_inplace"] = time_inplace(wl, torch, A, args.steps, args.warmup)
    if not profiling:
        result["roofline_score"] = time_score_test_time_shape(A, W, dev, torch)
    if not args.skip_cpu_baseline and not profiling:
        n_cpu, blas_threads = host_threads()
        times, parity, sample = wl.oracle_check(args.cpu_sample_rows)
        result["cpu_baseline"] = {"value": wl.T / sum(times.values()), "unit": "tokens/s", "cores": blas_threads,
                                  "host_logical_cpus": n_cpu, "kind": "oracle", "sample": sample,
                                  "stage_seconds_scaled": {k: round(v, 4) for k, v in times.items()},
                                  "parity_on_sample": parity}
    # the KV pools are not needed any more: free them before anything else is allocated
    wl.kv_src = wl.kv_dst = None
    torch.cuda.empty_cache()
    if args.vendor_gemm:
        result["vendor_gemm_reference"] = time_vendor_gemm(wl, torch)
    if args.mfma_probe or not (profiling or args.skip_mfma_probe):
        result["mfma_register_loop"] = time_mfma_probe(A, wl, torch)
    if args.extras:
        result["extras"] = time_extras(A, W, cfg, dev, torch, wl.lp_hidden, wl.lm_head, wl.targets, wl.cu)
    del wl
    torch.cuda.empty_cache()
    if not args.skip_all_configs and not profiling:
        result["all_configs"] = {}
        for name in ALL_WORKLOADS:
            if name != cfg.name:
                result["all_configs"][name] = run_config(A, W, torch, name, dev, args.config_steps, 1,
                                                         args.config_sample_rows)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
