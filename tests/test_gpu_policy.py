"""Parity of the stochastic pruning policy (histogram, calibration, Bernoulli prune) with the oracle."""
import numpy as np
import pytest
import torch

import oracle as O
from helpers import bits, npy, to_dev

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
Q_TOL = 1e-6      # fp64 arithmetic rounded to fp32 once
DELTA_TOL = 1e-9


@pytest.fixture(scope="module")
def A():
    import paper_2603_24840_amd as pkg
    pkg.lib()
    return pkg


@pytest.fixture(scope="module")
def W():
    from paper_2603_24840_amd import workloads
    return workloads


def f32(x):
    return float(np.float32(x))


@pytest.mark.parametrize("M,B", [(0, 128), (1, 128), (4096, 128), (100_000, 128), (777, 10), (5000, 1), (3000, 2048)])
def test_histogram_bit_exact(A, M, B):
    print("[case] histogram M=%d B=%d" % (M, B), flush=True)
    g = torch.Generator(device=DEV); g.manual_seed(M + B)
    s = torch.rand(max(M, 1), generator=g, device=DEV)[:M].contiguous()
    if M > 3:
        s[0] = 0.0; s[1] = 1.0; s[2] = 0.5
    lab = (torch.rand(max(M, 1), generator=g, device=DEV)[:M] < 0.3).to(torch.uint8).contiguous()
    c_pos, c_neg = A.arrol_histogram(s, lab, B)
    torch.cuda.synchronize()
    ref_pos, ref_neg = O.histogram(npy(s), npy(lab), B)
    assert np.array_equal(npy(c_pos), ref_pos) and np.array_equal(npy(c_neg), ref_neg)


@pytest.mark.parametrize("kappa,rho,lam,p_min,p_max,alpha", [(0.5, 0.5, 0.5, 0.05, 0.95, 1.0), (0.25, 0.5, 0.5, 0.1, 0.9, 0.5),
                                                             (0.75, 0.3, 2.0, 0.0, 1.0, 0.0), (0.5, 0.5, 0.0, 0.05, 0.95, 1.0),
                                                             (0.02, 0.5, 0.5, 0.05, 0.95, 1.0)])
def test_calibrate_matches_oracle(A, W, kappa, rho, lam, p_min, p_max, alpha):
    print("[case] calibrate kappa=%g rho=%g lambda=%g" % (kappa, rho, lam), flush=True)
    cfg = W.CONFIGS["llama1b"]
    s_buf, label, _, _ = W.policy_inputs(cfg, DEV)
    for B in (128, 16, 1000):
        # the histograms both sides calibrate on are the oracle's (the library's are checked bit for bit here too)
        cp_o, cn_o = O.histogram(npy(s_buf), npy(label), B)
        c_pos, c_neg = A.arrol_histogram(s_buf, label, B)
        pol = A.Policy(kappa, rho, lam, p_min, p_max, alpha)
        q_lut, p_lut, delta = A.arrol_calibrate(to_dev(cp_o, DEV, np.int64), to_dev(cn_o, DEV, np.int64), pol)
        torch.cuda.synchronize()
        assert np.array_equal(npy(c_pos), cp_o) and np.array_equal(npy(c_neg), cn_o)
        q_o, p_o, d_o = O.calibrate(cp_o, cn_o, f32(kappa), f32(rho), f32(lam), f32(p_min), f32(p_max), f32(alpha))
        assert np.max(np.abs(npy(q_lut) - q_o)) < Q_TOL
        assert np.max(np.abs(npy(p_lut) - p_o)) < Q_TOL
        if p_min < kappa < p_max:
            assert abs(float(delta[0]) - d_o) < DELTA_TOL
            w = O.bin_weights(cp_o, cn_o)
            assert abs(float(np.dot(w, npy(p_lut).astype(np.float64))) - f32(kappa)) < 1e-6   # E[p] = kappa


def test_calibrate_empty_buffers(A):
    z = torch.zeros(128, dtype=torch.int64, device=DEV)
    q_lut, p_lut, delta = A.arrol_calibrate(z, z.clone(), A.Policy(0.5, 0.5, 0.5, 0.05, 0.95, 1.0))
    torch.cuda.synchronize()
    assert np.all(npy(q_lut) == 0.5) and np.max(np.abs(npy(p_lut) - 0.5)) < Q_TOL and abs(float(delta[0])) < DELTA_TOL


@pytest.mark.parametrize("N", [0, 1, 63, 512, 1024, 1025, 32768, 100_001])
def test_prune_bernoulli_bit_exact(A, N):
    print("[case] prune_bernoulli N=%d" % N, flush=True)
    g = torch.Generator(device=DEV); g.manual_seed(N + 5)
    B = 128
    p_lut = torch.linspace(0.95, 0.05, B, device=DEV)
    s = torch.rand(max(N, 1), generator=g, device=DEV)[:N].contiguous()
    u = torch.rand(max(N, 1), generator=g, device=DEV)[:N].contiguous()
    out = A.arrol_prune_bernoulli(s, u, p_lut, want_p=True)
    torch.cuda.synchronize()
    p_o, keep_o, surv_o, n_o = O.prune_bernoulli(npy(s), npy(u), npy(p_lut))
    assert int(out["n_survivors"][0]) == n_o
    assert np.array_equal(npy(out["p"]), p_o) and np.array_equal(npy(out["keep_mask"]), keep_o)
    assert np.array_equal(npy(out["survivor_idx"])[:n_o], surv_o)
    assert np.all(npy(out["survivor_idx"])[n_o:] == -1)


def test_policy_end_to_end_feeds_compaction(A, W):
    """score buffer -> histogram -> calibrate -> Bernoulli prune -> compaction of the random-size survivor set.
    The oracle's chain runs from the inputs alone; its survival table, rounded to fp32, is what both sides'
    Bernoulli decisions are taken on (the library's own table agrees with it to 1e-6 and is used for the
    chain run, whose decisions can differ only where a uniform falls within that distance of p)."""
    cfg = W.shrink(W.CONFIGS["tiny"], n_prompts=16)
    s_buf, label, s_batch, uniforms = W.policy_inputs(cfg, DEV)
    pol = (0.5, 0.5, 0.5, 0.05, 0.95, 1.0)
    cp_o, cn_o = O.histogram(npy(s_buf), npy(label), 128)
    _, p_o, _ = O.calibrate(cp_o, cn_o, *[f32(x) for x in pol])
    p32 = p_o.astype(np.float32)
    _, keep_o, surv_o, n_o = O.prune_bernoulli(npy(s_batch), npy(uniforms), p32)

    c_pos, c_neg = A.arrol_histogram(s_buf, label, 128)
    _, p_lut, _ = A.arrol_calibrate(c_pos, c_neg, A.Policy(*pol))
    chain = A.arrol_prune_bernoulli(s_batch, uniforms, p_lut)                       # the library's own chain
    out = A.arrol_prune_bernoulli(s_batch, uniforms, to_dev(p32, DEV))              # decisions on the oracle's table
    kv, bt, sl, tok = W.compact_inputs(cfg, DEV)
    N = cfg.n_rollouts
    dst = torch.zeros((cfg.n_layers, 2, N * cfg.pages_per_rollout) + tuple(kv.shape[3:]), dtype=torch.bfloat16, device=DEV)
    cout = A.arrol_compact(kv, dst, bt, sl, tok, out["survivor_idx"])        # n_keep = N, tail entries are -1
    torch.cuda.synchronize()
    assert np.max(np.abs(npy(p_lut) - p_o)) < Q_TOL
    n = int(out["n_survivors"][0])
    assert abs(n / N - 0.5) < 0.15                                          # about kappa*N survive
    assert n == n_o and np.array_equal(npy(out["survivor_idx"])[:n], surv_o) and np.array_equal(npy(out["keep_mask"]), keep_o)
    # chain run: same decisions except where u is within the table tolerance of p
    p_of = p32[O.bin_index(npy(s_batch), 128)]
    sure = np.abs(npy(uniforms) - p_of) > 2 * Q_TOL
    assert np.array_equal(npy(chain["keep_mask"])[sure], keep_o[sure])
    ref = O.compact(bits(kv), npy(bt), npy(sl), npy(tok), surv_o, dst.shape[2])
    assert np.array_equal(bits(dst), ref["kv_dst"])
    assert int(cout["n_pages_used"][0]) == ref["n_pages_used"]
    assert np.array_equal(npy(cout["block_table_dst"])[:n], ref["block_table_dst"])
