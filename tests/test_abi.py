"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the
header declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "arrol.h")


@pytest.fixture(scope="module")
def pkg():
    import paper_2603_24840_amd as A
    if not os.path.exists(A.LIB_PATH):
        from paper_2603_24840_amd import build
        build.build(verbose=False)
    return A


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(arrol_[a-z_]+)\s*\(", text)))


def test_header_declares_the_five_stage_calls():
    names = declared_functions()
    for fn in ["arrol_score", "arrol_select", "arrol_compact", "arrol_logprob", "arrol_weighted_vote",
               "arrol_compact_workspace_bytes", "arrol_logprob_workspace_bytes", "arrol_version",
               "arrol_error_string", "arrol_histogram", "arrol_calibrate",
               "arrol_prune_bernoulli", "arrol_compact_static", "arrol_compact_inplace", "arrol_compact_inplace_workspace_bytes",
               "arrol_score_mlp", "arrol_score_mlp_workspace_bytes", "arrol_score_grad", "arrol_score_grad_workspace_bytes", "arrol_adamw_step", "arrol_score_mlp_grad",
               "arrol_score_mlp_grad_workspace_bytes", "arrol_token_confidence",
               "arrol_token_confidence_workspace_bytes", "arrol_trace_confidence",
               "arrol_trace_confidence_workspace_bytes", "arrol_grpo_advantage", "arrol_grpo_objective",
               "arrol_grpo_objective_workspace_bytes"]:
        assert fn in names


def test_library_exports_every_declared_symbol(pkg):
    handle = ctypes.CDLL(pkg.LIB_PATH)
    for fn in declared_functions():
        assert hasattr(handle, fn), fn


def test_binding_covers_every_declared_symbol(pkg):
    from paper_2603_24840_amd import binding
    assert sorted(binding._SIGNATURES) == declared_functions()


def test_version_and_error_strings(pkg):
    assert pkg.version() == 200
    assert pkg.error_string(0) == "ok"
    for code in (-1, -2, -3, -99):
        assert pkg.error_string(code)


def test_workspace_queries_are_pure_host_arithmetic(pkg):
    assert pkg.arrol_compact_workspace_bytes(0) >= 4
    assert pkg.arrol_compact_workspace_bytes(256) >= 257 * 4
    assert pkg.arrol_logprob_workspace_bytes(0, 100, 64) == 0
    small = pkg.arrol_logprob_workspace_bytes(2048, 4096, 256)
    big = pkg.arrol_logprob_workspace_bytes(294912, 128256, 2048)
    assert small >= 2048 * 12 and big >= 294912 * 12 and big % 256 == 0


def test_bad_arguments_are_rejected_on_the_host(pkg):
    L = pkg.lib()
    fake = ctypes.c_void_p(0x1000)      # never dereferenced: validation fails first
    # select: K > G, G > 64, K < 1, rho outside [0,1]
    assert L.arrol_select(fake, 4, 8, 9, 0.5, fake, fake, None) == -1
    assert L.arrol_select(fake, 4, 65, 4, 0.5, fake, fake, None) == -1
    assert L.arrol_select(fake, 4, 8, 0, 0.5, fake, fake, None) == -1
    assert L.arrol_select(fake, 4, 8, 4, 1.5, fake, fake, None) == -1
    assert L.arrol_select(None, 4, 8, 4, 0.5, fake, fake, None) == -1
    assert L.arrol_select(None, 0, 8, 4, 0.5, None, None, None) == 0        # empty batch is a no-op
    # score: d not a multiple of 8, stride < d, misaligned base
    assert L.arrol_score(fake, 12, None, fake, 0.0, 4, 12, None, fake, None) == -1
    assert L.arrol_score(fake, 8, None, fake, 0.0, 4, 16, None, fake, None) == -1
    assert L.arrol_score(ctypes.c_void_p(0x1004), 16, None, fake, 0.0, 4, 16, None, fake, None) == -1
    assert L.arrol_score(None, 16, None, None, 0.0, 0, 16, None, None, None) == 0
    # logprob: bad d, missing workspace
    assert L.arrol_logprob(fake, fake, fake, 10, 100, 12, fake, None, 0, fake, 1 << 20, None) == -1
    assert L.arrol_logprob(fake, fake, fake, 10, 0, 16, fake, None, 0, fake, 1 << 20, None) == -1
    assert L.arrol_logprob(fake, fake, fake, 10, 100, 16, fake, None, -1, fake, 1 << 20, None) == -1     # n_splits < 0
    assert L.arrol_logprob(fake, fake, fake, 10, 100, 16, fake, None, 0, None, 0, None) == -2
    assert L.arrol_logprob(fake, fake, fake, 10, 100, 16, fake, None, 0, fake, 8, None) == -2
    # a workspace sized for 2 splits is too small for 8 (600 rows x 4500 vocabulary entries = 18 tiles)
    two = L.arrol_logprob_workspace_bytes(600, 4500, 64, 2)
    assert L.arrol_logprob_workspace_bytes(600, 4500, 64, 8) > two >= 600 * 2 * 12
    assert L.arrol_logprob(fake, fake, fake, 600, 4500, 64, fake, None, 8, fake, two, None) == -2
    assert L.arrol_logprob(None, None, None, 0, 100, 16, None, None, 0, None, 0, None) == 0
    # vote: C > 64, no answers
    assert L.arrol_weighted_vote(fake, fake, 3, 65, 4, fake, None, None) == -1
    assert L.arrol_weighted_vote(fake, fake, 3, 8, 0, fake, None, None) == -1
    # compact: geometry mismatch, chunk not a multiple of 16 bytes, overlap, workspace
    lay = pkg.KVLayout(2, 16, 2, 64, 128)
    other = pkg.KVLayout(2, 16, 2, 32, 128)
    odd = pkg.KVLayout(2, 1, 1, 4, 128)
    far = ctypes.c_void_p(0x4000_0000)
    args = (fake, fake, 4, None, 0, fake, 32, 16, fake, fake, None, fake, fake)
    assert L.arrol_compact(fake, lay, far, other, *args, fake, 1 << 20, None) == -1
    assert L.arrol_compact(fake, odd, far, odd, *args, fake, 1 << 20, None) == -1
    assert L.arrol_compact(fake, lay, fake, lay, *args, fake, 1 << 20, None) == -1      # overlapping pools
    assert L.arrol_compact(fake, lay, far, lay, *args, None, 0, None) == -2
    assert L.arrol_compact(fake, lay, far, lay, *args, fake, 4, None) == -2
    # the variant without a workspace: same checks, and more survivors than its fixed scratch holds
    sargs = (fake, fake, 4, None, 0, fake, 32, 16, fake, fake, None, fake, fake)
    assert L.arrol_compact_static(fake, lay, far, other, *sargs, None) == -1
    assert L.arrol_compact_static(fake, lay, fake, lay, *sargs, None) == -1
    big = (fake, fake, 4, None, 0, fake, 1 << 20, 16384, fake, fake, None, fake, fake)
    assert L.arrol_compact_static(fake, lay, far, lay, *big, None) == -2
    # MLP head: bad d, m < 1, null weights
    assert L.arrol_score_mlp(fake, 16, None, fake, None, fake, 0.0, 4, 12, 8, None, fake, None, 0, None) == -1
    assert L.arrol_score_mlp(fake, 16, None, fake, None, fake, 0.0, 4, 16, 0, None, fake, None, 0, None) == -1
    assert L.arrol_score_mlp(fake, 16, None, fake, None, None, 0.0, 4, 16, 8, None, fake, None, 0, None) == -1
    assert L.arrol_score_mlp(None, 16, None, None, None, None, 0.0, 0, 16, 8, None, None, None, 0, None) == 0
    # scratch of the multi-launch paths: partial scores per 32-unit block (small batches) or per 256-unit tile
    # (beyond 4,096 rows); none when d % 64 != 0 (one-launch tile kernel only)
    assert L.arrol_score_mlp_workspace_bytes(512, 2048, 512) >= 16 * 512 * 4
    assert L.arrol_score_mlp_workspace_bytes(512, 2056, 512) == 0
    assert L.arrol_score_mlp_workspace_bytes(32768, 4096, 512) >= 2 * 32768 * 4
    # head training: bad d, missing gradient output, workspace; optimizer: bad step / betas
    assert L.arrol_score_grad(fake, 16, None, fake, 0.0, fake, 4, 12, None, fake, None, fake, 1 << 20, None) == -1
    assert L.arrol_score_grad(fake, 16384, None, fake, 0.0, fake, 4, 16384, None, fake, None, fake, 1 << 20, None) == -1
    assert L.arrol_score_grad(fake, 16, None, fake, 0.0, fake, 4, 16, None, None, None, fake, 1 << 20, None) == -1
    assert L.arrol_score_grad(fake, 16, None, fake, 0.0, None, 4, 16, None, fake, None, fake, 1 << 20, None) == -1
    assert L.arrol_score_grad(fake, 16, None, fake, 0.0, fake, 4, 16, None, fake, None, None, 0, None) == -2
    assert L.arrol_score_grad(fake, 16, None, fake, 0.0, fake, 4, 16, None, fake, None, fake, 8, None) == -2
    assert L.arrol_score_grad_workspace_bytes(4, 16) >= (16 + 2) * 4
    assert L.arrol_adamw_step(fake, fake, fake, fake, 8, 0, 1e-3, 0.9, 0.999, 1e-8, 0.0, None, None) == -1
    assert L.arrol_adamw_step(fake, fake, fake, fake, 8, 1, 1e-3, 1.0, 0.999, 1e-8, 0.0, None, None) == -1
    assert L.arrol_adamw_step(fake, None, fake, fake, 8, 1, 1e-3, 0.9, 0.999, 1e-8, 0.0, None, None) == -1
    assert L.arrol_adamw_step(None, None, None, None, 0, 1, 1e-3, 0.9, 0.999, 1e-8, 0.0, None, None) == 0
    # MLP head gradient: bad d, m < 1, missing outputs, workspace missing / short / misaligned
    mg = lambda d, m, gw1, ws, nbytes, terms=1: L.arrol_score_mlp_grad(fake, 16, None, fake, None, fake, 0.0, fake, 4, d, m, None,
                                                                        gw1, fake, fake, None, terms, ws, nbytes, None)
    assert mg(12, 8, fake, fake, 1 << 24) == -1
    assert mg(16, 0, fake, fake, 1 << 24) == -1
    assert mg(16, 8, None, fake, 1 << 24) == -1
    assert mg(16, 8, fake, None, 0) == -2
    assert mg(16, 8, fake, fake, 256) == -2
    assert mg(16, 8, fake, ctypes.c_void_p(0x1010), 1 << 24) == -2
    assert mg(16, 8, fake, fake, 1 << 24, terms=0) == -1 and mg(16, 8, fake, fake, 1 << 24, terms=3) == -1
    assert L.arrol_score_mlp_grad_workspace_bytes(4, 16, 8, 1) >= 3 * 4 * 4 + 128 * (16 + 8) * 2
    # the two-term form holds a second delta^T and a second partial of dL/dW1
    assert L.arrol_score_mlp_grad_workspace_bytes(4, 16, 8, 2) >= L.arrol_score_mlp_grad_workspace_bytes(4, 16, 8, 1) + 128 * 8 * 2 + 8 * 16 * 4
    assert L.arrol_score_mlp_grad_workspace_bytes(4, 16, 8, 0) == 0 and L.arrol_score_mlp_grad_workspace_bytes(4, 16, 8, 3) == 0
    # trace confidence: bad d / V, null lse, workspace; aggregates: window < 1, percent outside [1, 100]
    assert L.arrol_token_confidence(fake, fake, fake, 4, 100, 12, fake, fake, 1 << 20, None) == -1
    assert L.arrol_token_confidence(fake, fake, fake, 4, 0, 16, fake, fake, 1 << 20, None) == -1
    assert L.arrol_token_confidence(fake, fake, None, 4, 100, 16, fake, fake, 1 << 20, None) == -1
    assert L.arrol_token_confidence(fake, fake, fake, 4, 100, 16, fake, None, 0, None) == -2
    assert L.arrol_token_confidence(fake, fake, fake, 4, 100, 16, fake, fake, 64, None) == -2
    assert L.arrol_token_confidence(None, None, None, 0, 100, 16, None, None, 0, None) == 0
    assert L.arrol_token_confidence_workspace_bytes(100, 16) >= 2 * 16 * 4
    assert L.arrol_trace_confidence(fake, fake, 10, 2, 0, 10, fake, fake, fake, fake, 1 << 20, None) == -1
    assert L.arrol_trace_confidence(fake, fake, 10, 2, 4, 0, fake, fake, fake, fake, 1 << 20, None) == -1
    assert L.arrol_trace_confidence(fake, fake, 10, 2, 4, 101, fake, fake, fake, fake, 1 << 20, None) == -1
    assert L.arrol_trace_confidence(fake, None, 10, 2, 4, 10, fake, fake, fake, fake, 1 << 20, None) == -1
    assert L.arrol_trace_confidence(fake, fake, 10, 2, 4, 10, fake, fake, fake, None, 0, None) == -2
    assert L.arrol_trace_confidence(fake, fake, 10, 2, 4, 10, fake, fake, fake, fake, 100, None) == -2
    assert L.arrol_trace_confidence(None, None, 0, 0, 4, 10, None, None, None, None, 0, None) == 0
    assert L.arrol_trace_confidence_workspace_bytes(10, 2) == 2 * 12 * 8
    # GRPO: ddof outside {0, 1}, negative eps, clip range / beta outside their domain, workspace
    assert L.arrol_grpo_advantage(fake, fake, 8, 2, 2, 0.0, fake, None, None) == -1
    assert L.arrol_grpo_advantage(fake, fake, 8, 2, 0, -1.0, fake, None, None) == -1
    assert L.arrol_grpo_advantage(fake, None, 8, 2, 0, 0.0, fake, None, None) == -1
    assert L.arrol_grpo_advantage(None, None, 0, 0, 0, 0.0, None, None, None) == 0
    assert L.arrol_grpo_objective(fake, fake, fake, 8, 2, fake, fake, 1.5, 0.2, 0.0, fake, None, None, fake, 64, None) == -1
    assert L.arrol_grpo_objective(fake, fake, fake, 8, 2, fake, fake, 0.2, -0.1, 0.0, fake, None, None, fake, 64, None) == -1
    assert L.arrol_grpo_objective(fake, fake, fake, 8, 2, fake, fake, 0.2, 0.2, -1.0, fake, None, None, fake, 64, None) == -1
    assert L.arrol_grpo_objective(fake, fake, fake, 8, 2, None, fake, 0.2, 0.2, 0.0, fake, None, None, fake, 64, None) == -1
    assert L.arrol_grpo_objective(fake, fake, fake, 8, 2, fake, fake, 0.2, 0.2, 0.0, fake, None, None, None, 0, None) == -2
    assert L.arrol_grpo_objective(fake, fake, fake, 8, 2, fake, fake, 0.2, 0.2, 0.0, fake, None, None, fake, 16, None) == -2
    assert L.arrol_grpo_objective_workspace_bytes(2) == 32
    # in-place compaction: bad geometry, missing / short workspace
    assert L.arrol_compact_inplace(fake, odd, fake, fake, 4, fake, 32, 16, fake, fake, fake, fake, None, fake, 1 << 20, None) == -1
    assert L.arrol_compact_inplace(fake, lay, fake, fake, 0, fake, 32, 16, fake, fake, fake, fake, None, fake, 1 << 20, None) == -1
    assert L.arrol_compact_inplace(fake, lay, fake, fake, 4, fake, 32, 16, fake, fake, fake, None, None, fake, 1 << 20, None) == -1
    assert L.arrol_compact_inplace(fake, lay, fake, fake, 4, fake, 32, 16, fake, fake, fake, fake, None, None, 0, None) == -2
    assert L.arrol_compact_inplace(fake, lay, fake, fake, 4, fake, 32, 16, fake, fake, fake, fake, None, fake, 64, None) == -2
    assert pkg.lib().arrol_compact_inplace_workspace_bytes(128) >= (4 * 128 + 2) * 4
    # stochastic policy: bin count out of range, null outputs, policy outside its domain
    assert L.arrol_histogram(fake, fake, 10, 0, fake, fake, None) == -1
    assert L.arrol_histogram(fake, fake, 10, 4096, fake, fake, None) == -1
    assert L.arrol_histogram(None, fake, 10, 128, fake, fake, None) == -1
    good = pkg.Policy(0.5, 0.5, 0.5, 0.05, 0.95, 1.0)
    assert L.arrol_calibrate(fake, fake, 128, pkg.Policy(1.5, 0.5, 0.5, 0.05, 0.95, 1.0), fake, fake, None, None) == -1
    assert L.arrol_calibrate(fake, fake, 128, pkg.Policy(0.5, 0.5, 0.5, 0.9, 0.1, 1.0), fake, fake, None, None) == -1
    assert L.arrol_calibrate(fake, fake, 128, pkg.Policy(0.5, 0.5, -1.0, 0.05, 0.95, 1.0), fake, fake, None, None) == -1
    assert L.arrol_calibrate(fake, fake, 0, good, fake, fake, None, None) == -1
    assert L.arrol_calibrate(None, fake, 128, good, fake, fake, None, None) == -1
    assert L.arrol_prune_bernoulli(fake, fake, -1, fake, 128, None, fake, fake, fake, None) == -1
    assert L.arrol_prune_bernoulli(fake, fake, 8, fake, 128, None, fake, fake, None, None) == -1
    assert L.arrol_prune_bernoulli(None, fake, 8, fake, 128, None, fake, fake, fake, None) == -1
    # MFMA rate probe: unknown shape, partial fragments, misaligned operands, workgroup count, null sink
    assert L.arrol_probe_mfma_rate(fake, 512, fake, 512, 8, 4, 1, fake, None, None) == -1
    assert L.arrol_probe_mfma_rate(fake, 500, fake, 512, 16, 4, 1, fake, None, None) == -1
    assert L.arrol_probe_mfma_rate(fake, 512, fake, 0, 16, 4, 1, fake, None, None) == -1
    assert L.arrol_probe_mfma_rate(ctypes.c_void_p(0x1008), 512, fake, 512, 16, 4, 1, fake, None, None) == -1
    assert L.arrol_probe_mfma_rate(fake, 512, fake, 512, 16, 0, 1, fake, None, None) == -1
    assert L.arrol_probe_mfma_rate(fake, 512, fake, 512, 32, 4, -1, fake, None, None) == -1
    assert L.arrol_probe_mfma_rate(fake, 512, fake, 512, 32, 4, 1, None, None, None) == -1


def test_binding_refuses_cpu_tensors(pkg):
    import torch
    h = torch.zeros(4, 16, dtype=torch.bfloat16)
    with pytest.raises((TypeError, ValueError)):
        pkg.arrol_score(h, torch.zeros(16))
    with pytest.raises(ValueError):
        pkg.arrol_select(torch.zeros(8), 1, 8, 4)


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: `bench.py --gpus N` with N > 1 exits with a message that says so."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode == 2
    assert "ONE GPU" in res.stderr and "--gpus 2" in res.stderr
    assert res.stdout.strip() == ""


def test_binding_argument_counts_match_the_header(pkg):
    """Every prototype in include/arrol.h has as many parameters as its ctypes signature in the binding."""
    from paper_2603_24840_amd import binding
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    protos = re.findall(r"\b(arrol_[a-z_]+)\s*\(([^;{]*?)\)\s*;", text, flags=re.S)
    assert len(protos) == len(binding._SIGNATURES)
    for name, params in protos:
        params = " ".join(params.split())
        n = 0 if params in ("", "void") else params.count(",") + 1
        assert n == len(binding._SIGNATURES[name][1]), (name, n, len(binding._SIGNATURES[name][1]))
