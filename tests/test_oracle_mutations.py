"""Do the pins have teeth?  Each case plants ONE plausible mistake in a copy of the oracle's source (a dropped
term, a wrong sign or index, a swapped operand, an off-by-one), loads the copy as a module and runs the pins of
that function against it: at least one pin must fail.  Everything here runs on the CPU, on the oracle only."""
import importlib.util
import inspect
import os
import sys
import types

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_SRC = os.path.join(os.path.dirname(HERE), "oracle", "arrol_oracle.py")

# (pins to run: substring of the test names, text in the oracle, its mutated form)
MUTANTS = [
    ("score", "s[i] = math.fsum(h[i] * w64) + float(bias)", "s[i] = math.fsum(h[i] * w64)"),
    ("score", "q[i] = 1.0 / (1.0 + math.exp(-s[i]))", "q[i] = 1.0 / (1.0 + math.exp(s[i]))"),
    ("score", "q[i] = e / (1.0 + e)", "q[i] = 1.0 / (1.0 + e)"),
    ("bf16", "<< np.uint32(16)", "<< np.uint32(15)"),
    ("quantis", "np.rint(scaled)", "np.floor(scaled)"),
    ("select", "dev = abs(rest - R * (n - 1))", "dev = abs(rest - R * n)"),
    ("select", "if best_dev is None or dev < best_dev:", "if best_dev is None or dev <= best_dev:"),
    ("select", "rest = sum(k[i] for i in live if i != j)", "rest = sum(k[i] for i in live)"),
    ("select", "while len(live) > K:", "while len(live) > K + 1:"),
    ("select", "surv[g * K + r] = g * G + j", "surv[g * K + r] = j"),
    ("compact", "kv_dst[layer, c, base + p] = kv_src[layer, c, sp]", "kv_dst[layer, c, base + p] = kv_src[layer, c, p]"),
    ("compact", "base += n_pages", "base += ppr"),
    ("compact", "n_pages = -(-int(seq_len_src[src]) // page_tokens)", "n_pages = int(seq_len_src[src]) // page_tokens"),
    ("compact", "tok_dst[r, :] = tokens_src[src, :]", "tok_dst[r, :] = tokens_src[r, :]"),
    ("logprob", "logp[t0:t0 + step] = z[np.arange(z.shape[0]), targets[t0:t0 + step]] - l",
     "logp[t0:t0 + step] = z[np.arange(z.shape[0]), targets[t0:t0 + step]] + l"),
    ("logprob", "l = m + np.log(np.exp(z - m[:, None]).sum(axis=1))", "l = np.log(np.exp(z - m[:, None]).sum(axis=1))"),
    ("logprob", "        z = h @ W.T\n        m = z.max(axis=1)\n", "        z = h @ W.T[::-1]\n        m = z.max(axis=1)\n"),
    ("vote", "rank2.append(2 * below + equal)", "rank2.append(2 * below)"),
    ("vote", "below = sum(1 for j in range(C) if q[u, j] < q[u, i])", "below = sum(1 for j in range(C) if q[u, j] > q[u, i])"),
    ("vote", "if best is None or tally[u, a] > tally[u, best]:", "if best is None or tally[u, a] >= tally[u, best]:"),
    ("bin", "return np.minimum(B - 1, np.maximum(0, b))", "return np.maximum(0, b)"),
    ("histogram", "        if lab[k]:\n            c_pos[b[k]] += 1\n        else:\n            c_neg[b[k]] += 1",
     "        if lab[k]:\n            c_neg[b[k]] += 1\n        else:\n            c_pos[b[k]] += 1"),
    ("posterior", "like_pos = (c_pos + alpha) / (n_pos + alpha * B)", "like_pos = (c_pos + alpha) / (n_pos + alpha)"),
    ("posterior", "den = num + (1.0 - pi) * like_neg", "den = num + pi * like_neg"),
    ("survival", "return np.clip(kappa + delta + lam * (rho - q), p_min, p_max)", "return np.clip(kappa + delta + lam * (q - rho), p_min, p_max)"),
    ("survival", "        if float(np.dot(w, p_of(mid))) < kappa:\n            lo = mid\n        else:\n            hi = mid",
     "        if float(np.dot(w, p_of(mid))) < kappa:\n            hi = mid\n        else:\n            lo = mid"),
    ("prune_bernoulli", "if u[i] < p[i]:", "if u[i] > p[i]:"),
    ("inplace", "holes = [p for p in range(n_live) if p not in live]", "holes = [p for p in range(n_live) if p not in live][::-1]"),
    ("inplace", "movers = sorted(p for p in live if p >= n_live)", "movers = sorted(p for p in live if p > n_live)"),
    ("inplace", "bt_dst[r, p] = new_page[page]", "bt_dst[r, p] = page"),
    ("score_mlp", "act = np.where(pre > 0.0, pre, 0.0)\n        s[i] = math.fsum(act * w2) + float(b2)", "act = pre\n        s[i] = math.fsum(act * w2) + float(b2)"),
    ("score_mlp", "pre = W1 @ h[i] + b1\n        act = np.where(pre > 0.0, pre, 0.0)\n        s[i]", "pre = W1 @ h[i]\n        act = np.where(pre > 0.0, pre, 0.0)\n        s[i]"),
    ("score_ce", "terms.append(-(y[i] * _log_sigmoid(s) + (1.0 - y[i]) * _log_sigmoid(-s)))\n    return math.fsum(terms) / n\n\n\ndef score_ce_grad",
     "terms.append(-(y[i] * _log_sigmoid(-s) + (1.0 - y[i]) * _log_sigmoid(s)))\n    return math.fsum(terms) / n\n\n\ndef score_ce_grad"),
    ("score_ce", "r[i] = q - y[i]", "r[i] = y[i] - q"),
    ("score_ce", "    return score_ce(hidden_bits, w, bias, labels), grad_w, math.fsum(r) / n", "    return score_ce(hidden_bits, w, bias, labels), grad_w, math.fsum(r)"),
    ("adamw", "m_hat = m / (1.0 - beta1 ** step)", "m_hat = m"),
    ("adamw", "v = beta2 * v + (1.0 - beta2) * g * g", "v = beta2 * v + (1.0 - beta2) * g"),
    ("adamw", "p = p - lr * (m_hat / (np.sqrt(v_hat) + eps) + weight_decay * p)", "p = p - lr * (m_hat / (np.sqrt(v_hat) + eps)) - weight_decay * p"),
    ("token_confidence", "out[t] = -math.fsum(z - lse)", "out[t] = math.fsum(z - lse)"),
    ("token_confidence", "lse = m + math.log(math.fsum(np.exp(z - m)))\n        out[t]", "lse = math.log(math.fsum(np.exp(z - m)))\n        out[t]"),
    ("trace_confidence", "for k in range(L - w + 1))", "for k in range(L - w))"),
    ("trace_confidence", "m = max(1, (len(vals) * int(bottom_percent) + 99) // 100)", "m = max(1, (len(vals) * int(bottom_percent)) // 100)"),
    ("trace_confidence", "wmin[i] = vals[0]", "wmin[i] = vals[-1]"),
    ("grpo", "std = math.sqrt(math.fsum(dev * dev) / (n - ddof)) if n - ddof > 0 else 0.0", "std = math.fsum(dev * dev) / (n - ddof) if n - ddof > 0 else 0.0"),
    ("grpo", "clipped = min(max(ratio, 1.0 - eps_low), 1.0 + eps_high) * adv[i]", "clipped = min(max(ratio, 1.0 - eps_high), 1.0 + eps_low) * adv[i]"),
    ("grpo", "tok.append(min(plain, clipped) - beta * kl)", "tok.append(max(plain, clipped) - beta * kl)"),
    ("grpo", "kl = math.exp(u) - u - 1.0", "kl = math.exp(u) - 1.0"),
    ("grpo", "grad[t] = d / (L * G * n_groups)", "grad[t] = d / (L * n_groups)"),
    ("grpo", "d = plain if plain <= clipped else 0.0", "d = plain"),
    ("mlp_grad", "delta = np.where(pre > 0.0, r * w2, 0.0)", "delta = r * w2"),
    ("mlp_grad", "gw2 += r * act", "gw2 += r * pre"),
    ("mlp_grad", "gW1 += np.outer(delta, h[i])", "gW1 += np.outer(delta, h[i]) * 0.5"),
    ("compact", "src_of_dst[r] = src", "src_of_dst[r] = r"),
    ("compact", "sl_dst[r] = seq_len_src[src]", "sl_dst[r] = n_pages * page_tokens"),
    ("compact", "bt_dst[r, p] = base + p", "bt_dst[r, p] = sp"),
    ("select", "R = quantise(np.array([rho], dtype=np.float32))[0]", "R = quantise(np.array([0.5], dtype=np.float32))[0]"),
    ("select", "keep[g * G + j] = 1", "keep[g * G + r] = 1"),
    ("vote", "tally[u, ans[u, i]] += rank2[i]", "tally[u, ans[u, i]] += 1"),
    ("vote", "equal = sum(1 for j in range(C) if j != i and q[u, j] == q[u, i])", "equal = sum(1 for j in range(C) if q[u, j] == q[u, i])"),
    ("posterior", "pi = 0.5 if n_pos + n_neg == 0 else n_pos / (n_pos + n_neg)", "pi = 0.5"),
    ("posterior", "num = pi * like_pos", "num = like_pos"),
    ("survival", "lo, hi = p_min - kappa - lam, p_max - kappa + lam", "lo, hi = 0.0, p_max - kappa + lam"),
    ("calibrate", "p, delta = survival_lut(q, bin_weights(c_pos, c_neg), kappa, rho, lam, p_min, p_max)",
     "p, delta = survival_lut(q, bin_weights(c_neg, c_neg), kappa, rho, lam, p_min, p_max)"),
    ("inplace", "sl_dst[r] = seq_len_src[s]\n        src_of_dst[r] = s", "sl_dst[r] = seq_len_src[r]\n        src_of_dst[r] = s"),
    ("inplace", "kv[:, :, hole] = kv[:, :, mover]", "kv[:, :, mover] = kv[:, :, hole]"),
    ("adamw", "m = beta1 * m + (1.0 - beta1) * g", "m = beta1 * m + g"),
    ("adamw", "v_hat = v / (1.0 - beta2 ** step)", "v_hat = v / (1.0 - beta2)"),
    ("score_mlp", "s[i] = math.fsum(act * w2) + float(b2)", "s[i] = math.fsum(act * w2)"),
    ("mlp_grad", "gb1 += delta", "gb1 += r * w2"),
    ("mlp_grad", "r = (q - y[i]) / n\n        delta", "r = (q - y[i])\n        delta"),
    ("trace_confidence", "mean[i] = math.fsum(x) / L", "mean[i] = math.fsum(x) / max(L, window)"),
    ("trace_confidence", "w = min(int(window), L)", "w = int(window)"),
    ("grpo", "mean = math.fsum(x) / n\n        dev = x - mean", "mean = 0.5\n        dev = x - mean"),
    ("grpo", "u = lr[t] - lp[t]", "u = lp[t] - lr[t]"),
    ("grpo", "seq_terms.append(math.fsum(tok) / L)", "seq_terms.append(math.fsum(tok))"),
]


def load_mutant(old, new):
    src = open(ORACLE_SRC).read()
    assert src.count(old) >= 1, "mutation site not found in the oracle: %r" % old[:60]
    mod = types.ModuleType("oracle_mutant")
    mod.__file__ = ORACLE_SRC
    exec(compile(src.replace(old, new, 1), ORACLE_SRC, "exec"), mod.__dict__)
    mod.arrol_oracle = mod
    return mod


@pytest.fixture(scope="module")
def pins():
    spec = importlib.util.spec_from_file_location("pins_under_mutation", os.path.join(HERE, "test_oracle_pins.py"))
    mod = importlib.util.module_from_spec(spec)
    sys.path.insert(0, HERE)
    spec.loader.exec_module(mod)
    return mod


@pytest.mark.parametrize("case", range(len(MUTANTS)))
def test_a_planted_mistake_fails_a_pin(pins, case):
    keyword, old, new = MUTANTS[case]
    tests = [(n, f) for n, f in vars(pins).items()
             if n.startswith("test_") and keyword in n and callable(f) and not inspect.signature(f).parameters]
    assert tests, "no pin named *%s*" % keyword
    saved = pins.O
    pins.O = load_mutant(old, new)
    failed = []
    try:
        for name, fn in tests:
            try:
                fn()
            except pytest.skip.Exception:
                continue
            except Exception:          # a failed assertion, or the mutant breaking down outright
                failed.append(name)
    finally:
        pins.O = saved
    assert failed, "no pin among %s notices: %s -> %s" % ([n for n, _ in tests], old[:70], new[:70])
