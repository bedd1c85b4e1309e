"""Do the GPU parity tests have teeth?  A mistake is planted in a COPY OF THE ORACLE (never in a kernel: every
launch here is the ordinary, correct one) and the parity test of that stage is run against the copy: it must
report a mismatch.  This shows that the seeded inputs reach the code paths where the two sides could differ
(ties, ragged tails, last partial pages, clipped tokens...) and that the tolerances are not too loose."""
import importlib

import pytest
import torch

from test_oracle_mutations import load_mutant

pytestmark = pytest.mark.gpu

# (test module, test function, call arguments after the fixtures, text in the oracle, mutated form)
CASES = [
    ("test_gpu_random", "test_select_random_sweep", (), "if best_dev is None or dev < best_dev:", "if best_dev is None or dev <= best_dev:"),
    ("test_gpu_random", "test_select_random_sweep", (), "np.rint(scaled)", "np.floor(scaled)"),
    ("test_gpu_random", "test_vote_random_sweep", (), "rank2.append(2 * below + equal)", "rank2.append(2 * below)"),
    ("test_gpu_random", "test_vote_random_sweep", (), "if best is None or tally[u, a] > tally[u, best]:", "if best is None or tally[u, a] >= tally[u, best]:"),
    ("test_gpu_random", "test_compact_random_sweep", (), "n_pages = -(-int(seq_len_src[src]) // page_tokens)", "n_pages = int(seq_len_src[src]) // page_tokens"),
    ("test_gpu_random", "test_compact_inplace_random_sweep", (), "movers = sorted(p for p in live if p >= n_live)", "movers = sorted((p for p in live if p >= n_live), reverse=True)"),
    ("test_gpu_random", "test_prune_bernoulli_random_sweep", (), "return np.minimum(B - 1, np.maximum(0, b))", "return np.minimum(B - 1, np.maximum(0, b - 1))"),
    ("test_gpu_parity", "test_logprob_ragged_shapes", (257, 4097, 128), "l = m + np.log(np.exp(z - m[:, None]).sum(axis=1))", "l = m + np.log(np.exp(z - m[:, None])[:, :-1].sum(axis=1))"),
    ("test_gpu_parity", "test_logprob_ragged_shapes", (700, 2049, 320), "z = h @ W.T\n        m = z.max(axis=1)", "z = (h @ W.T) * (1.0 + 2e-4)\n        m = z.max(axis=1)"),
    ("test_gpu_parity", "test_score_matches_oracle", (1000, 2048), "s[i] = math.fsum(h[i] * w64) + float(bias)", "s[i] = math.fsum(h[i][:-1] * w64[:-1]) + float(bias)"),
    ("test_gpu_grpo", "test_objective_matches_oracle_ragged", (0.2, 0.28, 0.04), "d = plain if plain <= clipped else 0.0", "d = plain"),
    ("test_gpu_grpo", "test_objective_matches_oracle_ragged", (0.2, 0.28, 0.04), "clipped = min(max(ratio, 1.0 - eps_low), 1.0 + eps_high) * adv[i]", "clipped = min(max(ratio, 1.0 - eps_high), 1.0 + eps_low) * adv[i]"),
    ("test_gpu_confidence", "test_trace_confidence_ragged_batch", (64, 10), "m = max(1, (len(vals) * int(bottom_percent) + 99) // 100)", "m = max(1, (len(vals) * int(bottom_percent)) // 100)"),
    ("test_gpu_train", "test_score_grad_matches_oracle", (300, 1024), "r[i] = q - y[i]", "r[i] = q - 0.999 * y[i]"),
]


@pytest.fixture(scope="module")
def A():
    import paper_2603_24840_amd as pkg
    pkg.lib()
    return pkg


@pytest.fixture(scope="module")
def W():
    from paper_2603_24840_amd import workloads
    return workloads


@pytest.mark.parametrize("case", range(len(CASES)))
def test_parity_test_notices_a_mistake_planted_in_the_oracle(A, W, case):
    import inspect
    mod_name, fn_name, args, old, new = CASES[case]
    print("[case] teeth %s::%s %s" % (mod_name, fn_name, new[:50].replace("\n", " ")), flush=True)
    mod = importlib.import_module(mod_name)
    fn = getattr(mod, fn_name)
    fixtures = {"A": A, "W": W}
    lead = [fixtures[p] for p in inspect.signature(fn).parameters if p in fixtures]
    fn(*lead, *args)                      # the real oracle: the parity test passes
    saved = mod.O
    mod.O = load_mutant(old, new)
    try:
        with pytest.raises(AssertionError):
            fn(*lead, *args)
    finally:
        mod.O = saved
        torch.cuda.synchronize()
