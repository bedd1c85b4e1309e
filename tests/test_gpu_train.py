"""Parity of the quality-head training calls (cross-entropy loss + gradient, AdamW) with the oracle."""
import numpy as np
import pytest
import torch

import oracle as O
from helpers import bits, npy

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
# fp32 sums of N terms (|r_i h_ic| <= ~5) in a tree of depth N/grid + log: error ~ 1e-7 * sqrt(N) * 5 / N
# relative to a mean of magnitude <= 1; the bound below leaves two orders of margin at every size tested.
GRAD_ATOL, GRAD_RTOL = 2e-6, 2e-5
LOSS_RTOL = 2e-6


@pytest.fixture(scope="module")
def A():
    import paper_2603_24840_amd as pkg
    pkg.lib()
    return pkg


@pytest.fixture(scope="module")
def W():
    from paper_2603_24840_amd import workloads
    return workloads


def check_grad(A, hidden, w, bias, labels, row_index=None):
    loss, gw, gb = A.arrol_score_grad(hidden, w, bias, labels, row_index=row_index)
    torch.cuda.synchronize()
    hb = bits(hidden)
    if row_index is not None:
        hb = hb[npy(row_index)]
    loss_o, gw_o, gb_o = O.score_ce_grad(hb, npy(w), np.float32(bias), npy(labels))
    assert abs(float(loss) - loss_o) <= LOSS_RTOL * max(1.0, abs(loss_o)), (float(loss), loss_o)
    err = np.abs(npy(gw).astype(np.float64) - gw_o)
    assert np.all(err <= GRAD_ATOL + GRAD_RTOL * np.abs(gw_o)), float(err.max())
    assert abs(float(gb) - gb_o) <= GRAD_ATOL + GRAD_RTOL * abs(gb_o)
    return loss, gw, gb


@pytest.mark.parametrize("n,d", [(1, 8), (7, 24), (64, 512), (65, 520), (300, 1024), (513, 2048), (200, 3072),
                                 (130, 4096), (70, 8192), (90, 5000 // 8 * 8)])
def test_score_grad_matches_oracle(A, W, n, d):
    print("[case] score_grad n=%d d=%d" % (n, d), flush=True)
    cfg = W.shrink(W.CONFIGS["tiny"], d=d)
    hidden, w, _, labels = W.head_training_inputs(cfg, DEV, n_rows=n)
    check_grad(A, hidden, w * 3.0, 0.25, labels)


def test_score_grad_row_index_strided_rows_and_soft_labels(A, W):
    print("[case] score_grad row_index/strided/soft", flush=True)
    cfg = W.shrink(W.CONFIGS["tiny"], d=256)
    big, w, _, _ = W.head_training_inputs(cfg, DEV, n_rows=400)
    wide = torch.zeros(400, 320, dtype=torch.bfloat16, device=DEV)
    wide[:, :256] = big
    view = wide[:, :256]                                   # row stride 320 elements
    g = torch.Generator(device=DEV); g.manual_seed(3)
    idx = torch.randint(0, 400, (150,), generator=g, device=DEV, dtype=torch.int64)
    soft = torch.rand(150, generator=g, device=DEV)
    check_grad(A, view, w, -0.5, soft, row_index=idx)


def test_score_grad_many_rows_uses_every_workgroup_and_is_reproducible(A, W):
    print("[case] score_grad n=70000 d=128", flush=True)
    cfg = W.shrink(W.CONFIGS["tiny"], d=128)
    hidden, w, _, labels = W.head_training_inputs(cfg, DEV, n_rows=70_000)   # > 1024 workgroups * 64 rows
    l1, g1, b1 = check_grad(A, hidden, w * 2.0, 0.0, labels)
    l2, g2, b2 = A.arrol_score_grad(hidden, w * 2.0, 0.0, labels)
    torch.cuda.synchronize()
    assert torch.equal(g1, g2) and torch.equal(l1, l2) and torch.equal(b1, b2)


def test_score_grad_saturated_logits_and_empty_batch(A):
    print("[case] score_grad saturated / empty", flush=True)
    hidden = torch.full((2, 8), 16.0, dtype=torch.bfloat16, device=DEV)
    w = torch.full((8,), 8.0, device=DEV)
    labels = torch.tensor([1.0, 0.0], device=DEV)
    loss, gw, gb = A.arrol_score_grad(hidden, w, 0.0, labels)
    torch.cuda.synchronize()
    assert float(loss) == 512.0 and torch.all(gw == 8.0) and float(gb) == 0.5
    loss, gw, gb = A.arrol_score_grad(hidden[:0], w, 0.0, labels[:0])
    torch.cuda.synchronize()
    assert float(loss) == 0.0 and torch.all(gw == 0.0) and float(gb) == 0.0


def test_score_grad_full_training_shape(A, W):
    """The head's update at the benchmark configuration: every rollout of a step, d = 2048."""
    cfg = W.CONFIGS["llama1b"]
    print("[case] score_grad full n=%d d=%d" % (cfg.n_rollouts, cfg.d), flush=True)
    hidden, w, _, labels = W.head_training_inputs(cfg, DEV)
    check_grad(A, hidden, w, 0.0, labels)


@pytest.mark.parametrize("n", [1, 255, 4096, 1_000_003])
def test_adamw_matches_oracle_over_three_steps(A, n):
    print("[case] adamw n=%d" % n, flush=True)
    g = torch.Generator(device=DEV); g.manual_seed(n)
    p = torch.randn(n, generator=g, device=DEV)
    m = torch.zeros(n, device=DEV)
    v = torch.zeros(n, device=DEV)
    pb = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    hp = dict(lr=1e-2, beta1=0.9, beta2=0.99, eps=1e-8, weight_decay=0.05)
    for t in (1, 2, 3):
        grad = torch.randn(n, generator=g, device=DEV) * (10.0 ** (t - 2))
        p0, m0, v0 = npy(p), npy(m), npy(v)
        A.arrol_adamw_step(p, grad, m, v, t, param_bf16=pb, **hp)
        torch.cuda.synchronize()
        f = lambda x: float(np.float32(x))
        p_o, m_o, v_o = O.adamw_step(p0, npy(grad), m0, v0, t, f(1e-2), f(0.9), f(0.99), f(1e-8), f(0.05))
        g64 = np.abs(npy(grad).astype(np.float64))
        # m adds two rounded products that may cancel: the error scales with the operands, not the result
        assert np.all(np.abs(npy(m) - m_o) <= 4e-7 * (np.abs(m0) + g64)), "m"
        assert np.all(np.abs(npy(v) - v_o) <= 1e-6 * v_o), "v"
        assert np.all(np.abs(npy(p) - p_o) <= 1e-7 + 2e-6 * np.abs(p_o)), "p"
        # the bf16 copy is the round-to-nearest-even image of the fp32 parameters the call stored
        from helpers import f32_to_bf16_bits
        assert np.array_equal(bits(pb), f32_to_bf16_bits(npy(p)))


def test_head_training_loop_reduces_the_loss(A, W):
    """End to end: gradient + AdamW for a few steps lowers the cross-entropy on the same batch, and the
    trajectory stays on the oracle's (loss after five steps within 1e-4 relative)."""
    print("[case] training loop", flush=True)
    cfg = W.shrink(W.CONFIGS["tiny"], d=64)
    hidden, w, _, labels = W.head_training_inputs(cfg, DEV, n_rows=512)
    w = w.clone()
    b = torch.zeros(1, device=DEV)
    m, v = torch.zeros_like(w), torch.zeros_like(w)
    w_o, m_o, v_o = npy(w).astype(np.float64), np.zeros(64), np.zeros(64)
    hb, y = bits(hidden), npy(labels)
    losses = []
    for t in range(1, 6):
        loss, gw, _ = A.arrol_score_grad(hidden, w, 0.0, labels)
        A.arrol_adamw_step(w, gw, m, v, t, lr=5e-2)
        losses.append(float(loss))
        lo, gwo, _ = O.score_ce_grad(hb, w_o.astype(np.float32), 0.0, y)
        w_o, m_o, v_o = O.adamw_step(w_o.astype(np.float32), gwo.astype(np.float32), m_o, v_o, t, float(np.float32(5e-2)))
        assert abs(losses[-1] - lo) <= 1e-4 * lo
    assert losses[-1] < losses[0]


# ----------------------------------------------------------------------------- MLP head
def mlp_case(n, d, m, seed):
    g = torch.Generator(device=DEV); g.manual_seed(seed)
    hidden = torch.randn(n, d, generator=g, device=DEV).to(torch.bfloat16)
    w1 = (torch.randn(m, d, generator=g, device=DEV) * d ** -0.5).to(torch.bfloat16)
    b1 = torch.randn(m, generator=g, device=DEV) * 0.1
    w2 = torch.randn(m, generator=g, device=DEV) * m ** -0.5
    labels = (torch.rand(n, generator=g, device=DEV) < 0.4).to(torch.float32)
    return hidden, w1, b1, w2, labels


def check_mlp_grad(A, hidden, w1, b1, w2, b2, labels, row_index=None, delta_terms=1):
    out = A.arrol_score_mlp_grad(hidden, w1, b1, w2, b2, labels, row_index=row_index, delta_terms=delta_terms)
    torch.cuda.synchronize()
    hb = bits(hidden)
    if row_index is not None:
        hb = hb[npy(row_index)]
    m = w1.shape[0]
    b1n = np.zeros(m, np.float32) if b1 is None else npy(b1)
    loss_o, gW1_o, gb1_o, gw2_o, gb2_o = O.score_mlp_ce_grad(hb, bits(w1), b1n, npy(w2), np.float32(b2), npy(labels))
    n = hb.shape[0]
    # quantities the tolerances are built from (float64, from the same inputs)
    H = O.bf16_bits_to_f64(hb)
    pre = H @ O.bf16_bits_to_f64(bits(w1)).T + b1n.astype(np.float64)             # [n, m]
    s, q = O.score_mlp(hb, bits(w1), b1n, npy(w2), np.float32(b2))
    r = (q - npy(labels).astype(np.float64)) / n
    w2n = npy(w2).astype(np.float64)
    delta = np.abs(r[:, None] * w2n[None, :]) * (pre > 0)                          # |delta| [n, m]
    # a pre-activation within fp32 rounding of zero may gate differently in fp32 than in float64
    near = np.abs(pre) < 4e-6 * (np.abs(H) @ np.abs(O.bf16_bits_to_f64(bits(w1))).T + 1.0)
    flip = np.abs(r[:, None] * w2n[None, :]) * near
    F32 = 4e-6
    assert abs(float(out["loss"]) - loss_o) <= 1e-5 * max(1.0, abs(loss_o))
    assert abs(float(out["grad_b2"]) - gb2_o) <= F32 * np.sum(np.abs(r)) + 1e-9
    tol_b1 = F32 * delta.sum(axis=0) + flip.sum(axis=0) + 1e-9 * np.abs(w2n)
    assert np.all(np.abs(npy(out["grad_b1"]) - gb1_o) <= tol_b1)
    act = np.maximum(pre, 0.0)
    tol_w2 = F32 * (np.abs(r)[:, None] * act).sum(axis=0) + 1e-9 * act.mean(axis=0) + 1e-12
    assert np.all(np.abs(npy(out["grad_w2"]) - gw2_o) <= tol_w2)
    # dL/dW1: delta is rounded to bf16 (unit roundoff 2^-8, worst case summed; 2^-16 for the two-term form),
    # fp32 accumulation on top
    unit = 2.0 ** -8 if delta_terms == 1 else 2.0 ** -16
    bound = (unit + F32) * (delta.T @ np.abs(H)) + flip.T @ np.abs(H) + 1e-12
    err = np.abs(npy(out["grad_w1"]).astype(np.float64) - gW1_o)
    assert np.all(err <= bound), float((err / bound).max())
    # rounding errors average out: the error as a whole is far below the worst case
    if not near.any() and np.linalg.norm(gW1_o) > 0:
        assert np.linalg.norm(err) <= (2.0 ** -8 if delta_terms == 1 else 1e-5) * np.linalg.norm(gW1_o)
    return out


@pytest.mark.parametrize("n,d,m", [(1, 8, 1), (32, 256, 64), (130, 264, 100), (300, 1024, 257), (512, 2048, 512),
                                   (1500, 512, 300),
                                   (4500, 128, 300), (4097, 64, 7), (5000, 192, 512),      # beyond 4,096 rows: the ring-pipeline kernels
                                   (4200, 320, 70), (8195, 576, 260)])                     # ... more than one 256-column block of dL/dW1
def test_score_mlp_grad_matches_oracle(A, n, d, m):
    print("[case] score_mlp_grad n=%d d=%d m=%d" % (n, d, m), flush=True)
    hidden, w1, b1, w2, labels = mlp_case(n, d, m, seed=n + d + m)
    check_mlp_grad(A, hidden, w1, b1, w2 * 4.0, -0.125, labels)


@pytest.mark.parametrize("n,d,m", [(130, 264, 100),      # tile kernels (d not a multiple of 64)
                                   (300, 1024, 257),     # wavefront-per-block forward, in-place dL/dW1, one K split
                                   (512, 2048, 512),
                                   (2048, 256, 128),     # several K splits
                                   (4500, 128, 300)])    # ring-pipeline forward
def test_score_mlp_grad_two_term_delta_is_fp32_accurate(A, n, d, m):
    """delta_terms = 2: dL/dW1 within 1e-5 of the float64 oracle in norm (2^-8 for the one-term form), and
    strictly closer than the one-term result; everything else unchanged bit for bit."""
    print("[case] score_mlp_grad two-term n=%d d=%d m=%d" % (n, d, m), flush=True)
    hidden, w1, b1, w2, labels = mlp_case(n, d, m, seed=3 * n + d + m)
    o2 = check_mlp_grad(A, hidden, w1, b1, w2 * 4.0, -0.125, labels, delta_terms=2)
    o1 = A.arrol_score_mlp_grad(hidden, w1, b1, w2 * 4.0, -0.125, labels)
    torch.cuda.synchronize()
    for k in ("loss", "grad_b1", "grad_w2", "grad_b2"):
        assert torch.equal(o1[k], o2[k]), k
    _, gW1_o, _, _, _ = O.score_mlp_ce_grad(bits(hidden), bits(w1), npy(b1), npy(w2 * 4.0), np.float32(-0.125), npy(labels))
    e1 = np.linalg.norm(npy(o1["grad_w1"]).astype(np.float64) - gW1_o)
    e2 = np.linalg.norm(npy(o2["grad_w1"]).astype(np.float64) - gW1_o)
    assert e2 < 0.05 * e1, (e1, e2)


def test_score_mlp_grad_two_term_delta_gathered_rows(A):
    print("[case] score_mlp_grad two-term gathered", flush=True)
    hidden, w1, b1, w2, _ = mlp_case(200, 128, 96, seed=5)
    g = torch.Generator(device=DEV); g.manual_seed(8)
    idx = torch.randint(0, 200, (150,), generator=g, device=DEV, dtype=torch.int64)
    soft = torch.rand(150, generator=g, device=DEV)
    check_mlp_grad(A, hidden, w1, b1, w2, 0.0, soft, row_index=idx, delta_terms=2)


def test_score_mlp_grad_gathered_rows_no_bias_dead_units_and_empty_batch(A):
    print("[case] score_mlp_grad gathered / dead / empty", flush=True)
    hidden, w1, b1, w2, _ = mlp_case(200, 128, 96, seed=5)
    wide = torch.zeros(200, 160, dtype=torch.bfloat16, device=DEV)
    wide[:, :128] = hidden
    view = wide[:, :128]
    g = torch.Generator(device=DEV); g.manual_seed(6)
    idx = torch.randint(0, 200, (77,), generator=g, device=DEV, dtype=torch.int64)
    soft = torch.rand(77, generator=g, device=DEV)
    check_mlp_grad(A, view, w1, None, w2, 0.0, soft, row_index=idx)
    dead = b1.clone()
    dead[::3] = -1e4                                   # a third of the units never fire
    out = check_mlp_grad(A, view, w1, dead, w2, 0.5, soft, row_index=idx)
    assert torch.all(out["grad_w1"][::3] == 0) and torch.all(out["grad_b1"][::3] == 0) and torch.all(out["grad_w2"][::3] == 0)
    out = A.arrol_score_mlp_grad(hidden[:0], w1, b1, w2, 0.0, soft[:0])
    torch.cuda.synchronize()
    assert float(out["loss"]) == 0.0 and float(out["grad_b2"]) == 0.0
    assert not out["grad_w1"].any() and not out["grad_b1"].any() and not out["grad_w2"].any()


def test_score_mlp_grad_large_batch_strided_rows_and_reproducible(A):
    """Ring-pipeline path on rows that are a view into a wider buffer (dL/dW1 contracts the hidden states in
    place, rollout-major); two calls give identical bits."""
    print("[case] score_mlp_grad n=4300 d=192 of 256 m=130 strided", flush=True)
    hidden, w1, b1, w2, labels = mlp_case(4300, 192, 130, seed=21)
    wide = torch.full((4300, 256), float("nan"), dtype=torch.bfloat16, device=DEV)   # what lies beside the rows is never read
    wide[:, :192] = hidden
    o1 = check_mlp_grad(A, wide[:, :192], w1, b1, w2 * 2.0, 0.25, labels)
    o2 = A.arrol_score_mlp_grad(wide[:, :192], w1, b1, w2 * 2.0, 0.25, labels)
    torch.cuda.synchronize()
    for k in o1:
        assert torch.equal(o1[k], o2[k]), k


def test_score_mlp_grad_is_reproducible_and_trains(A):
    """Two calls give identical bits; gradient + AdamW on all four parameter sets lowers the loss."""
    print("[case] score_mlp_grad reproducible / training loop", flush=True)
    hidden, w1, b1, w2, labels = mlp_case(2048, 256, 128, seed=9)          # three K splits
    o1 = A.arrol_score_mlp_grad(hidden, w1, b1, w2, 0.0, labels)
    o2 = A.arrol_score_mlp_grad(hidden, w1, b1, w2, 0.0, labels)
    torch.cuda.synchronize()
    for k in o1:
        assert torch.equal(o1[k], o2[k]), k
    master = w1.float().clone()
    params = [master.view(-1), b1.clone(), w2.clone()]
    state = [(torch.zeros_like(p), torch.zeros_like(p)) for p in params]
    w1_bf16 = w1.clone()
    losses = []
    for t in range(1, 9):
        out = A.arrol_score_mlp_grad(hidden, w1_bf16, params[1], params[2], 0.0, labels)
        losses.append(float(out["loss"]))
        grads = [out["grad_w1"].view(-1), out["grad_b1"], out["grad_w2"]]
        for k, (p, gk, (mk, vk)) in enumerate(zip(params, grads, state)):
            A.arrol_adamw_step(p, gk, mk, vk, t, lr=1e-2, param_bf16=w1_bf16.view(-1) if k == 0 else None)
    assert losses[-1] < losses[0] - 0.01, losses
