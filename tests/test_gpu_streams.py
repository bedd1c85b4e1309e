"""The five calls only enqueue work on the stream they are given: they run on a side stream while the
default stream is busy, and the whole step can be captured into a HIP graph and replayed on new inputs."""
import numpy as np
import pytest
import torch

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


class Step:
    """Pre-allocated buffers of one prune -> compact -> log-prob -> vote step on a reduced llama1b geometry."""

    def __init__(self, A, W, index):
        self.A = A
        cfg = W.shrink(W.CONFIGS["llama1b"], index=index, n_prompts=16, n_layers=2, vocab=8192, resp_lo=16, resp_hi=96,
                       vote_q=16, vote_c=8)
        self.cfg = cfg
        self.hidden, self.w, self.bias = W.score_inputs(cfg, DEV)
        self.kv_src, self.block_table, self.seq_len, self.tokens = W.compact_inputs(cfg, DEV)
        self.lp_hidden, self.lm_head, self.targets, _ = W.logprob_inputs(cfg, DEV, T=cfg.n_keep * 40)
        _, self.answer_id = W.vote_inputs(cfg, DEV)
        N, Nk, ppr, T = cfg.n_rollouts, cfg.n_keep, cfg.pages_per_rollout, self.lp_hidden.shape[0]
        i32 = lambda *shape: torch.empty(shape, dtype=torch.int32, device=DEV)
        self.score = torch.empty(N, device=DEV)
        self.prob = torch.empty(N, device=DEV)
        self.keep = torch.empty(N, dtype=torch.uint8, device=DEV)
        self.surv = i32(Nk)
        self.kv_dst = torch.zeros((cfg.n_layers, 2, Nk * ppr) + tuple(self.kv_src.shape[3:]), dtype=torch.bfloat16,
                                  device=DEV)
        self.cout = dict(block_table_dst=i32(Nk, ppr), seq_len_dst=i32(Nk), tokens_dst=i32(Nk, self.tokens.shape[1]),
                         src_of_dst=i32(Nk), n_pages_used=torch.empty(1, dtype=torch.int64, device=DEV))
        self.cws = torch.empty(max(16, A.arrol_compact_workspace_bytes(Nk)), dtype=torch.uint8, device=DEV)
        self.logprob = torch.empty(T, device=DEV)
        self.lws = torch.empty(max(16, A.arrol_logprob_workspace_bytes(T, cfg.vocab, cfg.d)), dtype=torch.uint8,
                               device=DEV)
        self.winner = i32(cfg.vote_q)

    def enqueue(self, stream=None):
        A, cfg = self.A, self.cfg
        A.arrol_score(self.hidden, self.w, self.bias, out_score=self.score, out_prob=self.prob, stream=stream)
        A.arrol_select(self.prob, cfg.n_prompts, cfg.G, cfg.K, cfg.rho, out_keep=self.keep, out_survivors=self.surv,
                       stream=stream)
        A.arrol_compact(self.kv_src, self.kv_dst, self.block_table, self.seq_len, self.tokens, self.surv,
                        out=self.cout, workspace=self.cws, stream=stream)
        A.arrol_logprob(self.lp_hidden, self.lm_head, self.targets, out_logprob=self.logprob, workspace=self.lws,
                        stream=stream)
        A.arrol_weighted_vote(self.prob[:cfg.vote_q * cfg.vote_c], self.answer_id, cfg.vote_q, cfg.vote_c, cfg.vote_a,
                              out_winner=self.winner, stream=stream)

    def outputs(self):
        return [self.score, self.prob, self.keep, self.surv, self.kv_dst, self.logprob, self.winner] + \
            [v for v in self.cout.values() if v is not None]

    def snapshot(self):
        return [t.clone() for t in self.outputs()]

    def load_inputs_from(self, other):
        for name in ("hidden", "w", "kv_src", "block_table", "seq_len", "tokens", "lp_hidden", "lm_head", "targets",
                     "answer_id"):
            getattr(self, name).copy_(getattr(other, name))


def test_step_on_a_side_stream_matches_the_default_stream(A, W):
    print("[case] side stream", flush=True)
    ref = Step(A, W, 1)
    ref.enqueue()
    torch.cuda.synchronize()
    want = ref.snapshot()
    side = torch.cuda.Stream()                         # default priority
    st = Step(A, W, 1)
    torch.cuda.synchronize()
    busy = torch.randn(4096, 4096, device=DEV)
    for _ in range(4):
        busy = busy @ busy * 1e-4                      # keeps the default stream occupied meanwhile
    st.enqueue(stream=side)
    side.synchronize()
    for got, exp in zip(st.outputs(), want):
        assert torch.equal(got, exp)
    torch.cuda.synchronize()


def test_side_stream_calls_that_allocate_their_own_workspace(A, W):
    """With workspace=None the binding creates the scratch itself; it must belong to the stream the kernels run
    on, or the allocator could hand it to the default stream's work below while those kernels still use it."""
    print("[case] side stream, temporaries created by the binding", flush=True)
    st = Step(A, W, 2)
    cfg = st.cfg
    lp_ref = A.arrol_logprob(st.lp_hidden, st.lm_head, st.targets)
    out_ref = A.arrol_compact(st.kv_src, st.kv_dst, st.block_table, st.seq_len, st.tokens,
                              A.arrol_select(A.arrol_score(st.hidden, st.w, st.bias)[1], cfg.n_prompts, cfg.G, cfg.K)[1])
    torch.cuda.synchronize()
    kv_ref = st.kv_dst.clone()
    st.kv_dst.zero_()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()                         # default priority
    _, q = A.arrol_score(st.hidden, st.w, st.bias, stream=side)
    _, surv = A.arrol_select(q, cfg.n_prompts, cfg.G, cfg.K, stream=side)
    out = A.arrol_compact(st.kv_src, st.kv_dst, st.block_table, st.seq_len, st.tokens, surv, stream=side)
    lp = A.arrol_logprob(st.lp_hidden, st.lm_head, st.targets, stream=side)
    # default-stream work that allocates and overwrites memory of the sizes just dropped
    junk = [torch.full((A.arrol_logprob_workspace_bytes(st.lp_hidden.shape[0], cfg.vocab, cfg.d) // 4,), float("nan"),
                       device=DEV) for _ in range(4)]
    side.synchronize()
    assert torch.equal(lp, lp_ref)
    assert torch.equal(st.kv_dst.view(torch.int16), kv_ref.view(torch.int16))
    for k in out_ref:
        assert torch.equal(out[k], out_ref[k]), k
    del junk
    torch.cuda.synchronize()


def test_step_captured_in_a_graph_replays_on_new_inputs(A, W):
    print("[case] graph capture", flush=True)
    st = Step(A, W, 1)
    st.enqueue()                                       # warm-up outside the capture (one-time attribute set-up)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        st.enqueue()
    for index in (2, 3, 1, 4):
        fresh = Step(A, W, index)                      # new seeded inputs, eager reference
        fresh.enqueue()
        torch.cuda.synchronize()
        want = fresh.snapshot()
        st.load_inputs_from(fresh)
        for t in st.outputs():
            t.zero_() if t.dtype != torch.bfloat16 else t.fill_(0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, exp in zip(st.outputs(), want):
            assert torch.equal(got, exp), index
