"""Seeded synthetic inputs shaped like the paper's 1B-8B Qwen-3 / LLaMA-3.2 workloads.

Input generation only: nothing of the method's arithmetic lives here.  Both the HIP
path and the CPU oracle are fed from these generators (tensors are produced once, on the
requested device, and copied to the host for the oracle).  Where a generator squashes random
scores with torch.sigmoid it only shapes the distribution of a synthetic INPUT (probabilities
fed to the selection, labelled score buffers, reward labels); neither the library's nor the
oracle's scoring is involved.
"""
from dataclasses import dataclass, replace

import numpy as np
import torch

BASE_SEED = 260324840


@dataclass(frozen=True)
class Config:
    name: str
    index: int
    n_prompts: int          # B
    G: int                  # rollouts per prompt
    K: int                  # kept per prompt
    d: int                  # hidden size
    ckpt_len: int           # tokens in cache at the pruning checkpoint (L_detect)
    n_layers: int
    n_kv_heads: int
    head_dim: int
    page_tokens: int
    vocab: int
    resp_lo: int            # survivor response lengths ~ U[resp_lo, resp_hi]
    resp_hi: int
    vote_q: int             # test-time vote: questions, candidates, answer ids
    vote_c: int
    vote_a: int
    rho: float = 0.5

    @property
    def n_rollouts(self):
        return self.n_prompts * self.G

    @property
    def n_keep(self):
        return self.n_prompts * self.K

    @property
    def pages_per_rollout(self):
        return -(-self.ckpt_len // self.page_tokens)

    @property
    def chunk_bytes(self):
        return self.page_tokens * self.n_kv_heads * self.head_dim * 2


CONFIGS = {
    "tiny": Config("tiny", 0, 4, 8, 4, 256, 64, 2, 2, 64, 16, 4096, 128, 128, 1, 8, 4),
    "llama1b": Config("llama1b", 1, 64, 8, 4, 2048, 512, 16, 8, 64, 16, 128256, 256, 2048, 64, 8, 16),
    "qwen1p7b": Config("qwen1p7b", 2, 128, 8, 4, 2048, 1024, 28, 8, 128, 16, 151936, 512, 4096, 128, 8, 16),
    "llama3b": Config("llama3b", 3, 64, 16, 8, 3072, 1024, 28, 8, 128, 16, 128256, 512, 4096, 64, 16, 16),
    "qwen8b": Config("qwen8b", 4, 64, 16, 8, 4096, 1024, 36, 8, 128, 16, 151936, 1024, 8192, 512, 64, 16),
}


def shrink(cfg, **kw):
    """A copy of cfg with some fields replaced (used for reduced-size parity cases)."""
    return replace(cfg, **kw)


def _gen(cfg, stage, device):
    g = torch.Generator(device=device)
    g.manual_seed(BASE_SEED + 1000 * cfg.index + stage)
    return g


def randn_bf16(shape, gen, device, std=1.0, slab=1 << 26):
    """bf16 ~ N(0, std^2), generated in fp32 slabs to bound the temporary."""
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    flat = out.view(-1)
    n = flat.numel()
    for s in range(0, n, slab):
        e = min(n, s + slab)
        tmp = torch.randn(e - s, generator=gen, device=device, dtype=torch.float32)
        if std != 1.0:
            tmp.mul_(std)
        flat[s:e] = tmp.to(torch.bfloat16)
    return out


def score_inputs(cfg, device, n_rows=None):
    """Checkpoint hidden states [N, d] bf16 ~ N(0,1); head weights fp32 ~ N(0, 1/d); bias 0."""
    g = _gen(cfg, 1, device)
    n = cfg.n_rollouts if n_rows is None else n_rows
    hidden = randn_bf16((n, cfg.d), g, device)
    w = torch.randn(cfg.d, generator=g, device=device, dtype=torch.float32) * (cfg.d ** -0.5)
    return hidden, w, 0.0


def head_training_inputs(cfg, device, n_rows=None):
    """Labelled hidden states for one update of the quality head: hidden / head weights as in score_inputs;
    the reward label of a row is 1 with probability sigmoid(2 <w*, h>) for a hidden "true" direction w*,
    so labels correlate with the hidden state but the current head (w) does not yet predict them."""
    hidden, w, bias = score_inputs(cfg, device, n_rows)
    g = _gen(cfg, 9, device)
    w_true = torch.randn(cfg.d, generator=g, device=device, dtype=torch.float32) * (cfg.d ** -0.5)
    p_true = torch.sigmoid(2.0 * (hidden.float() @ w_true))
    labels = (torch.rand(hidden.shape[0], generator=g, device=device) < p_true).to(torch.float32)
    return hidden, w, bias, labels


def select_inputs(cfg, device):
    """Probabilities as the sigmoid of N(0,1) scores (what stage 1 yields at these shapes)."""
    g = _gen(cfg, 2, device)
    s = torch.randn(cfg.n_rollouts, generator=g, device=device, dtype=torch.float32)
    return torch.sigmoid(s)


def compact_inputs(cfg, device, extra_pages=0, ragged=False, n_layers=None):
    """Paged KV pool bf16 ~ N(0,1); block tables = one random permutation of all pages cut into
    rows; every rollout holds ckpt_len tokens (ragged=True draws lengths in [1, ckpt_len]);
    token ids uniform over the vocabulary."""
    g = _gen(cfg, 3, device)
    L = cfg.n_layers if n_layers is None else n_layers
    N, ppr = cfg.n_rollouts, cfg.pages_per_rollout
    P = N * ppr + extra_pages
    kv = randn_bf16((L, 2, P, cfg.page_tokens, cfg.n_kv_heads, cfg.head_dim), g, device)
    perm = torch.randperm(P, generator=g, device=device)[:N * ppr]
    block_table = perm.to(torch.int32).reshape(N, ppr).contiguous()
    if ragged:
        seq_len = torch.randint(1, cfg.ckpt_len + 1, (N,), generator=g, device=device, dtype=torch.int32)
    else:
        seq_len = torch.full((N,), cfg.ckpt_len, dtype=torch.int32, device=device)
    tokens = torch.randint(0, cfg.vocab, (N, cfg.ckpt_len), generator=g, device=device, dtype=torch.int32)
    return kv, block_table, seq_len, tokens


def response_lengths(cfg, device="cpu"):
    """Survivor response lengths, i.i.d. uniform integers in [resp_lo, resp_hi] (host tensor)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(BASE_SEED + 1000 * cfg.index + 4)
    return torch.randint(cfg.resp_lo, cfg.resp_hi + 1, (cfg.n_keep,), generator=g, dtype=torch.int64)


def logprob_inputs(cfg, device, T=None, vocab=None):
    """Packed survivor hidden states [T, d] bf16 ~ N(0,1), LM head [V, d] bf16 ~ N(0, 1/d),
    targets uniform over the vocabulary, cu_seqlens of the ragged survivors."""
    g = _gen(cfg, 5, device)
    lens = response_lengths(cfg)
    cu = torch.zeros(cfg.n_keep + 1, dtype=torch.int64)
    cu[1:] = torch.cumsum(lens, 0)
    total = int(cu[-1]) if T is None else T
    V = cfg.vocab if vocab is None else vocab
    lm_head = randn_bf16((V, cfg.d), g, device, std=cfg.d ** -0.5)
    hidden = randn_bf16((total, cfg.d), g, device)
    targets = torch.randint(0, V, (total,), generator=g, device=device, dtype=torch.int32)
    for row, value in edge_target_rows(total, V):
        targets[row] = value
    return hidden, lm_head, targets, cu


VOCAB_TILE = 256    # edge cases are planted on multiples of this (the vocabulary is processed in 256-row tiles)


def edge_target_rows(T, V):
    """(row, target) pairs written over the uniform targets so that every batch, whatever its size, holds the
    edge targets a check must see: 0, V-1, both sides of the first vocabulary-tile edge and of the last one."""
    last_edge = (V - 1) // VOCAB_TILE * VOCAB_TILE
    values = [0, V - 1, min(VOCAB_TILE - 1, V - 1), min(VOCAB_TILE, V - 1), max(last_edge - 1, 0), last_edge]
    if T < 8 * len(values):
        return []
    return [((k + 1) * T // (len(values) + 2), v) for k, v in enumerate(values)]


def logprob_check_rows(T, n, V, cu=None, seed=7):
    """Sorted row sample of size about n for comparing log-probs against the oracle: a seeded random draw
    plus the rows that must always be looked at - row 0, row T-1, both sides of the first token-tile edge,
    the first and last row of the first and last survivor (from cu_seqlens), and the rows that carry the
    planted edge targets."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    rows = set(torch.randperm(T, generator=g)[:max(0, n)].tolist())
    rows.update(r for r in (0, 1, T - 2, T - 1, VOCAB_TILE - 1, VOCAB_TILE) if 0 <= r < T)
    if cu is not None and len(cu) >= 2:
        c = [int(x) for x in cu]
        rows.update(r for r in (c[0], c[1] - 1, c[-2], c[-1] - 1) if 0 <= r < T)
    rows.update(r for r, _ in edge_target_rows(T, V))
    return torch.tensor(sorted(rows), dtype=torch.int64)


def bits(t):
    """bf16 torch tensor (any device) -> uint16 numpy array of its bit patterns (what the oracle takes)."""
    assert t.dtype == torch.bfloat16
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def npy(t):
    """torch tensor (any device) -> numpy array on the host."""
    return t.detach().cpu().numpy()


def vote_inputs(cfg, device):
    """Candidate hidden states for the quality head and answer ids uniform in [0, A)."""
    g = _gen(cfg, 6, device)
    n = cfg.vote_q * cfg.vote_c
    hidden = randn_bf16((n, cfg.d), g, device)
    answer_id = torch.randint(0, cfg.vote_a, (n,), generator=g, device=device, dtype=torch.int32)
    return hidden, answer_id


def policy_inputs(cfg, device, buffer_len=4096, n_bins=128):
    """Labelled score buffer for the stochastic policy: head scores ~ N(+0.8, 1) for rollouts that turned
    out correct and N(-0.8, 1) for the others (a head of about 80 % accuracy, as the paper reports),
    positives with probability 0.4, squashed by the sigmoid; plus the batch's own normalised scores and
    uniforms for the Bernoulli draws."""
    g = _gen(cfg, 7, device)
    label = (torch.rand(buffer_len, generator=g, device=device) < 0.4)
    raw = torch.randn(buffer_len, generator=g, device=device) + torch.where(label, 0.8, -0.8)
    s_buf = torch.sigmoid(raw).to(torch.float32)
    blabel = (torch.rand(cfg.n_rollouts, generator=g, device=device) < 0.4)
    s_batch = torch.sigmoid(torch.randn(cfg.n_rollouts, generator=g, device=device) + torch.where(blabel, 0.8, -0.8))
    uniforms = torch.rand(cfg.n_rollouts, generator=g, device=device, dtype=torch.float32)
    return s_buf, label.to(torch.uint8), s_batch.to(torch.float32), uniforms
