"""Parity of the GRPO advantage / clipped-ratio objective calls with the oracle."""
import numpy as np
import pytest
import torch

import oracle as O
from helpers import npy, to_dev

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RTOL = 2e-6        # fp64 arithmetic on both sides; the results are rounded to fp32 once (6e-8) and the
                   # per-rollout weight is passed as fp32 (6e-8); 2e-6 leaves margin for cancellation in J


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


def dev_i64(a):
    return torch.tensor(np.asarray(a, dtype=np.int64), device=DEV)


@pytest.mark.parametrize("sizes,ddof,eps", [([4] * 64, 0, 0.0), ([8, 1, 0, 3, 64, 65, 200, 2], 0, 0.0),
                                            ([5, 7, 1, 16], 1, 0.0), ([4, 4, 6], 0, 1e-6)])
def test_advantage_matches_oracle(A, sizes, ddof, eps):
    print("[case] grpo_advantage sizes=%s ddof=%d" % (sizes[:8], ddof), flush=True)
    off = np.concatenate([[0], np.cumsum(sizes)])
    N = int(off[-1])
    g = torch.Generator(device=DEV); g.manual_seed(N + ddof)
    reward = (torch.rand(N, generator=g, device=DEV) < 0.4).to(torch.float32)
    reward[:sizes[0]] = 1.0                                  # first group: all equal -> zero advantage
    if len(sizes) > 5:
        reward[off[5]:off[6]] = torch.randn(sizes[5], generator=g, device=DEV)   # real-valued rewards
    adv, wgt = A.arrol_grpo_advantage(reward, dev_i64(off), ddof=ddof, eps=eps)
    torch.cuda.synchronize()
    ref = O.grpo_advantage(npy(reward), off, ddof=ddof, eps=f32(eps))
    assert np.all(np.abs(npy(adv) - ref) <= RTOL * np.abs(ref)), float(np.abs(npy(adv) - ref).max())
    assert np.all(npy(adv)[:sizes[0]] == 0.0)
    for gi, n in enumerate(sizes):
        if n:
            assert np.all(npy(wgt)[off[gi]:off[gi + 1]] == np.float32(1.0 / (n * len(sizes))))


def run_objective(A, lens, sizes, seed, eps_low=0.2, eps_high=0.2, beta=0.0, drift=0.3):
    cu = np.concatenate([[0], np.cumsum(lens)])
    off = np.concatenate([[0], np.cumsum(sizes)])
    assert off[-1] == len(lens)
    T = int(cu[-1])
    g = torch.Generator(device=DEV); g.manual_seed(seed)
    logp_ref = -torch.rand(max(T, 1), generator=g, device=DEV)[:T] * 4
    logp = logp_ref + torch.randn(max(T, 1), generator=g, device=DEV)[:T] * drift
    reward = (torch.rand(len(lens), generator=g, device=DEV) < 0.5).to(torch.float32)
    # advantages: the oracle's, rounded to the interface's fp32, feed both sides; the per-rollout weights
    # 1/(group size * groups) are what arrol_grpo_advantage hands to the objective (checked in the test above)
    adv_o = O.grpo_advantage(npy(reward), off).astype(np.float32)
    adv = to_dev(adv_o, DEV)
    _, wgt = A.arrol_grpo_advantage(reward, dev_i64(off))
    J, grad, n_clip = A.arrol_grpo_objective(logp, logp_ref, dev_i64(cu), adv, wgt, eps_low, eps_high, beta)
    torch.cuda.synchronize()
    Jo, go, co = O.grpo_objective(npy(logp), npy(logp_ref), cu, adv_o, off, f32(eps_low), f32(eps_high), f32(beta))
    scale = max(abs(Jo), float(np.mean(np.abs(adv_o))) if len(lens) else 0.0, 1e-30)
    assert abs(float(J) - Jo) <= RTOL * scale, (float(J), Jo)
    assert int(n_clip) == co
    err = np.abs(npy(grad).astype(np.float64) - go)
    assert np.all(err <= RTOL * np.abs(go) + 1e-30), float(err.max())
    return float(J), co, T


@pytest.mark.parametrize("beta", [0.0, 0.04])
@pytest.mark.parametrize("eps_low,eps_high", [(0.2, 0.2), (0.2, 0.28)])
def test_objective_matches_oracle_ragged(A, eps_low, eps_high, beta):
    print("[case] grpo_objective eps=(%g,%g) beta=%g" % (eps_low, eps_high, beta), flush=True)
    lens = [1, 2, 0, 255, 256, 257, 1000, 3, 64, 700, 5, 9]
    J, n_clip, T = run_objective(A, lens, [4, 2, 6], seed=int(beta * 100) + 7, eps_low=eps_low, eps_high=eps_high,
                                 beta=beta)
    assert 0 < n_clip < T


def test_objective_on_policy_and_degenerate_inputs(A):
    print("[case] grpo_objective on-policy / empty", flush=True)
    run_objective(A, [10, 20, 30, 40], [4], seed=3, drift=0.0)          # ratio 1: nothing clipped
    run_objective(A, [0, 0, 0], [3], seed=4)                            # only empty rollouts
    J, grad, n_clip = A.arrol_grpo_objective(torch.empty(0, device=DEV), torch.empty(0, device=DEV), dev_i64([0]),
                                             torch.empty(0, device=DEV), torch.empty(0, device=DEV))
    torch.cuda.synchronize()
    assert float(J) == 0.0 and int(n_clip) == 0


def test_objective_benchmark_shape(A, W):
    """llama1b survivors: 64 groups of K = 4 rollouts with the benchmark's response-length mix."""
    cfg = W.CONFIGS["llama1b"]
    lens = W.response_lengths(cfg).numpy().tolist()
    print("[case] grpo_objective llama1b n=%d T=%d" % (len(lens), sum(lens)), flush=True)
    run_objective(A, lens, [cfg.K] * (len(lens) // cfg.K), seed=11, beta=0.01)
