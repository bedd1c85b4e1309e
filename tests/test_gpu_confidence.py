"""Parity of the trace-confidence calls (token confidence from the log-prob pass, trace aggregates)."""
import numpy as np
import pytest
import torch

import oracle as O
from helpers import bits, npy, to_dev

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
AGG_RTOL = 1e-10   # fp64 prefix sums of magnitude L*|H| differenced per window: ~L/w * 2^-52 relative


def conf_tol(V, ref):
    """H_t = V*lse - <h, colsum W>: lse carries the log-prob kernel's fp32 error (<= 4e-6 observed bound,
    well inside the 2e-3 bar per log-probability), multiplied by V; the fp32 result adds 1e-6 relative."""
    return V * 4e-6 + 2e-6 * np.abs(ref)


@pytest.fixture(scope="module")
def A():
    import paper_2603_24840_amd as pkg
    pkg.lib()
    return pkg


@pytest.fixture(scope="module")
def W():
    from paper_2603_24840_amd import workloads
    return workloads


@pytest.mark.parametrize("T,V,d", [(1, 1, 8), (5, 2, 8), (70, 300, 64), (33, 1000, 72), (129, 5000, 256),
                                   (64, 777, 2048), (40, 2500, 4096), (17, 513, 8200)])
def test_token_confidence_matches_oracle(A, W, T, V, d):
    print("[case] token_confidence T=%d V=%d d=%d" % (T, V, d), flush=True)
    cfg = W.shrink(W.CONFIGS["tiny"], d=d, vocab=V)
    hidden, lm_head, targets, _ = W.logprob_inputs(cfg, DEV, T=T, vocab=V)
    _, lse = A.arrol_logprob(hidden, lm_head, targets, want_lse=True)
    conf = A.arrol_token_confidence(hidden, lm_head, lse)                     # the library's chain
    ref = O.token_confidence(bits(hidden), bits(lm_head))
    _, lse_o = O.logprob(bits(hidden), bits(lm_head), npy(targets))
    lse32 = lse_o.astype(np.float32)
    conf2 = A.arrol_token_confidence(hidden, lm_head, to_dev(lse32, DEV))     # the stage on the oracle's lse
    torch.cuda.synchronize()
    # stage parity: only the fp32 rounding of lse (times V), the fp32 dot product and the fp32 result remain
    tol2 = V * np.abs(lse32 - lse_o) + 1e-5 * np.sqrt(V) + 2e-6 * np.abs(ref)
    err2 = np.abs(npy(conf2).astype(np.float64) - ref)
    assert np.all(err2 <= tol2), (float((err2 / tol2).max()), float(err2.max()))
    err = np.abs(npy(conf).astype(np.float64) - ref)
    assert np.all(err <= conf_tol(V, ref)), (float(err.max()), float(np.abs(ref).max()))


def test_token_confidence_peaked_distribution(A):
    """Large logits: the confidence is dominated by V*lse; checks the fp64 combination of the two terms."""
    print("[case] token_confidence peaked", flush=True)
    g = torch.Generator(device=DEV); g.manual_seed(5)
    hidden = (torch.randn(24, 64, generator=g, device=DEV) * 4).to(torch.bfloat16)
    lm_head = (torch.randn(900, 64, generator=g, device=DEV)).to(torch.bfloat16)
    targets = torch.zeros(24, dtype=torch.int32, device=DEV)
    ref = O.token_confidence(bits(hidden), bits(lm_head))
    _, lse_o = O.logprob(bits(hidden), bits(lm_head), npy(targets))
    lse32 = lse_o.astype(np.float32)
    conf = A.arrol_token_confidence(hidden, lm_head, to_dev(lse32, DEV))      # the stage on the oracle's lse
    torch.cuda.synchronize()
    tol = 900 * np.abs(lse32 - lse_o) + 2e-6 * np.abs(ref) + 1e-3
    assert np.all(np.abs(npy(conf).astype(np.float64) - ref) <= tol)


def test_token_confidence_full_vocabulary_sampled_tokens(A, W):
    """Benchmark geometry (V = 128,256, d = 2048) on a few hundred tokens; the oracle checks a sample."""
    cfg = W.CONFIGS["llama1b"]
    T = 700
    print("[case] token_confidence full vocab T=%d" % T, flush=True)
    hidden, lm_head, targets, _ = W.logprob_inputs(cfg, DEV, T=T)
    _, lse = A.arrol_logprob(hidden, lm_head, targets, want_lse=True)
    conf = A.arrol_token_confidence(hidden, lm_head, lse)
    torch.cuda.synchronize()
    rows = np.random.default_rng(1).choice(T, 12, replace=False)
    ref = O.token_confidence(bits(hidden)[rows], bits(lm_head))
    err = np.abs(npy(conf).astype(np.float64)[rows] - ref)
    assert np.all(err <= conf_tol(cfg.vocab, ref)), float(err.max())


def run_trace(A, conf, lens, window, pct=10):
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int64, device=DEV)
    mean, wmin, bottom = A.arrol_trace_confidence(conf, cu, window, pct)
    torch.cuda.synchronize()
    mo, wo, bo = O.trace_confidence(npy(conf), npy(cu), window, pct)
    for got, want, name in ((mean, mo, "mean"), (wmin, wo, "min"), (bottom, bo, "bottom")):
        got = npy(got)
        assert np.array_equal(np.isnan(got), np.isnan(want)), name
        ok = ~np.isnan(want)
        assert np.all(np.abs(got[ok] - want[ok]) <= AGG_RTOL * np.abs(want[ok]) + 1e-300), (name, got, want)


@pytest.mark.parametrize("window,pct", [(1, 10), (4, 10), (64, 10), (2048, 10), (100000, 10), (16, 1), (16, 100), (7, 33)])
def test_trace_confidence_ragged_batch(A, window, pct):
    print("[case] trace_confidence window=%d pct=%d" % (window, pct), flush=True)
    lens = [0, 1, 2, 3, 63, 64, 65, 255, 256, 257, 2047, 2048, 2049, 5000, 0, 9, 4100]
    g = torch.Generator(device=DEV); g.manual_seed(window * 101 + pct)
    T = int(sum(lens))
    # magnitudes of the real signal: V*ln V ~ 1.5e6 with a spread of a few hundred
    conf = (1.5e6 + 400.0 * torch.randn(T, generator=g, device=DEV)).to(torch.float32)
    run_trace(A, conf, lens, window, pct)


def test_trace_confidence_ties_constant_and_negative_values(A):
    print("[case] trace_confidence ties / negative", flush=True)
    lens = [300, 300, 50]
    conf = torch.cat([torch.full((300,), 7.0, device=DEV),
                      torch.tensor(np.tile([3.0, -2.0, -2.0, 5.0, 0.0, -0.0], 50), dtype=torch.float32, device=DEV),
                      -torch.arange(50, device=DEV, dtype=torch.float32)])
    for window, pct in ((1, 10), (3, 50), (6, 10), (2, 100)):
        run_trace(A, conf, lens, window, pct)


def test_trace_confidence_real_length_mix(A, W):
    """The benchmark's response-length mix (llama1b survivors), window 2048, bottom 10 %."""
    cfg = W.CONFIGS["llama1b"]
    lens = W.response_lengths(cfg).numpy()
    print("[case] trace_confidence llama1b lengths n=%d T=%d" % (len(lens), int(lens.sum())), flush=True)
    g = torch.Generator(device=DEV); g.manual_seed(9)
    conf = (1.5e6 + 400.0 * torch.randn(int(lens.sum()), generator=g, device=DEV)).to(torch.float32)
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int64, device=DEV)
    mean, wmin, bottom = A.arrol_trace_confidence(conf, cu, 2048, 10)
    torch.cuda.synchronize()
    pick = np.random.default_rng(2).choice(len(lens), 6, replace=False)
    c = npy(conf)
    for i in pick:
        lo, hi = int(npy(cu)[i]), int(npy(cu)[i + 1])
        mo, wo, bo = O.trace_confidence(c[lo:hi], [0, hi - lo], 2048, 10)
        for got, want in ((mean, mo), (wmin, wo), (bottom, bo)):
            assert abs(float(got[i]) - want[0]) <= AGG_RTOL * abs(want[0])


def test_confidence_chain_end_to_end(A, W):
    """logprob -> token confidence -> trace aggregates on a ragged batch against the oracle chain."""
    print("[case] confidence chain", flush=True)
    cfg = W.shrink(W.CONFIGS["tiny"], d=128, vocab=640)
    lens = [40, 7, 0, 130, 64]
    T = sum(lens)
    hidden, lm_head, targets, _ = W.logprob_inputs(cfg, DEV, T=T, vocab=640)
    _, lse = A.arrol_logprob(hidden, lm_head, targets, want_lse=True)
    conf = A.arrol_token_confidence(hidden, lm_head, lse)
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int64, device=DEV)
    mean, wmin, bottom = A.arrol_trace_confidence(conf, cu, 16, 10)
    torch.cuda.synchronize()
    ref_conf = O.token_confidence(bits(hidden), bits(lm_head))
    mo, wo, bo = O.trace_confidence(ref_conf, npy(cu), 16, 10)
    tol = 640 * 4e-6 + 2e-6 * np.nanmax(np.abs(mo))
    for got, want in ((mean, mo), (wmin, wo), (bottom, bo)):
        got = npy(got)
        assert np.array_equal(np.isnan(got), np.isnan(want))
        ok = ~np.isnan(want)
        assert np.all(np.abs(got[ok] - want[ok]) <= tol)
