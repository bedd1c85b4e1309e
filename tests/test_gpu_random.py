"""Seeded random sweeps of the integer / byte stages (select, vote, both compactions, Bernoulli prune) over
shapes, tie patterns and index layouts; every case is compared bit for bit with the oracle."""
import numpy as np
import pytest
import torch

import oracle as O
from helpers import bits, npy, bf16_tensor_from_bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def A():
    import paper_2603_24840_amd as pkg
    pkg.lib()
    return pkg


def random_probs(rng, n):
    mode = rng.integers(0, 7)
    if mode == 6:
        return (rng.integers(0, 64, n) * 0.5 * 2.0 ** -30).astype(np.float32)   # half-way between fixed-point codes
    if mode == 0:
        p = rng.random(n)
    elif mode == 1:
        p = rng.integers(0, 5, n) / 4.0                       # heavy exact ties
    elif mode == 2:
        p = rng.integers(0, 2, n).astype(np.float64)          # only 0 and 1
    elif mode == 3:
        p = 0.5 + (rng.integers(-3, 4, n)) * 2.0 ** -24       # neighbours in fp32 around 1/2
    elif mode == 4:
        p = rng.beta(0.2, 0.2, n)                             # piled up at both ends
    else:
        p = np.full(n, rng.random())
    return p.astype(np.float32)


def test_select_random_sweep(A):
    rng = np.random.default_rng(20260324)
    for case in range(160):
        G = int(rng.integers(1, 65))
        K = int(rng.integers(1, G + 1))
        n_groups = int(rng.integers(1, 41))
        rho = float(rng.choice([0.0, 0.25, 0.5, 0.75, 1.0, rng.random()]))
        p = random_probs(rng, n_groups * G)
        keep, surv = A.arrol_select(torch.from_numpy(p).to(DEV), n_groups, G, K, rho)
        torch.cuda.synchronize()
        keep_o, surv_o = O.select(p, n_groups, G, K, float(np.float32(rho)))
        assert np.array_equal(npy(keep), keep_o) and np.array_equal(npy(surv), surv_o), (case, n_groups, G, K, rho)


def test_vote_random_sweep(A):
    rng = np.random.default_rng(20260325)
    for case in range(120):
        Q, C, n_ans = int(rng.integers(1, 51)), int(rng.integers(1, 65)), int(rng.integers(1, 41))
        p = random_probs(rng, Q * C)
        ans = rng.integers(0, n_ans, Q * C).astype(np.int32)
        win, tally = A.arrol_weighted_vote(torch.from_numpy(p).to(DEV), torch.from_numpy(ans).to(DEV), Q, C, n_ans,
                                           want_tally=True)
        torch.cuda.synchronize()
        win_o, tally_o = O.weighted_vote(p, ans, Q, C, n_ans)
        assert np.array_equal(npy(win), win_o) and np.array_equal(npy(tally), tally_o), (case, Q, C, n_ans)


def random_pool(rng):
    """A paged KV pool with ragged rollouts: returns geometry and host arrays."""
    L = int(rng.integers(1, 4))
    H = int(rng.choice([1, 2, 4]))
    hd = int(rng.choice([8, 16, 32, 64]))
    pt = int(rng.choice([1, 2, 4, 16]))
    while (pt * H * hd * 2) % 16:
        pt *= 2
    n_src = int(rng.integers(1, 25))
    ppr = int(rng.integers(1, 7))
    seq_len = rng.integers(0, ppr * pt + 1, n_src).astype(np.int32)
    extra = int(rng.integers(0, 9))
    P = n_src * ppr + extra
    table = rng.permutation(P)[:n_src * ppr].reshape(n_src, ppr).astype(np.int32)
    kv = rng.integers(0, 1 << 16, (L, 2, P, pt, H, hd), dtype=np.uint16)
    kv[(kv & 0x7F80) == 0x7F80] = 0x3C00            # no NaN / Inf patterns: contents are compared as bits anyway
    max_len = int(rng.integers(1, 40))
    tokens = rng.integers(0, 50000, (n_src, max_len)).astype(np.int32)
    n_keep = int(rng.integers(0, n_src + 1))
    surv = np.sort(rng.permutation(n_src)[:n_keep]).astype(np.int32)
    return kv, table, seq_len, tokens, surv, pt


def test_compact_random_sweep(A):
    rng = np.random.default_rng(20260326)
    for case in range(40):
        kv, table, seq_len, tokens, surv, pt = random_pool(rng)
        need = int(sum(-(-int(seq_len[s]) // pt) for s in surv))
        n_dst = need + int(rng.integers(0, 4))
        if n_dst == 0:
            n_dst = 1
        poison = 0x7FC1
        dst = torch.full((kv.shape[0], 2, n_dst) + kv.shape[3:], poison, dtype=torch.int16, device=DEV).view(torch.bfloat16)
        out = A.arrol_compact(bf16_tensor_from_bits(kv, DEV), dst, torch.from_numpy(table).to(DEV),
                              torch.from_numpy(seq_len).to(DEV), torch.from_numpy(tokens).to(DEV),
                              torch.from_numpy(surv).to(DEV))
        torch.cuda.synchronize()
        ref = O.compact(kv, table, seq_len, tokens, surv, n_dst, fill=poison)
        tag = (case, kv.shape, len(surv))
        assert np.array_equal(bits(dst), ref["kv_dst"]), tag
        for k in ("block_table_dst", "seq_len_dst", "tokens_dst", "src_of_dst"):
            assert np.array_equal(npy(out[k]), ref[k]), (tag, k)
        assert int(out["n_pages_used"][0]) == ref["n_pages_used"], tag


def test_compact_inplace_random_sweep(A):
    rng = np.random.default_rng(20260327)
    for case in range(40):
        kv, table, seq_len, _, surv, pt = random_pool(rng)
        if rng.random() < 0.3 and len(surv):
            surv = surv.copy()
            surv[int(rng.integers(0, len(surv)))] = -1          # an empty slot among the survivors
        dev_kv = bf16_tensor_from_bits(kv, DEV)
        ref_kv = kv.copy()
        ref = O.compact_inplace(ref_kv, table, seq_len, surv)
        out = A.arrol_compact_inplace(dev_kv, torch.from_numpy(table).to(DEV), torch.from_numpy(seq_len).to(DEV),
                                      torch.from_numpy(surv).to(DEV))
        torch.cuda.synchronize()
        tag = (case, kv.shape, len(surv))
        assert int(out["n_pages_used"][0]) == ref["n_pages_used"] and int(out["n_moved"][0]) == ref["n_moved"], tag
        for k in ("block_table_dst", "seq_len_dst", "src_of_dst"):
            assert np.array_equal(npy(out[k]), ref[k]), (tag, k)
        assert np.array_equal(bits(dev_kv), ref_kv), tag


def test_prune_bernoulli_random_sweep(A):
    rng = np.random.default_rng(20260328)
    for case in range(60):
        N, B = int(rng.integers(0, 3000)), int(rng.choice([1, 2, 16, 128, 1000, 2048]))
        s = random_probs(rng, max(N, 1))[:N]
        u = rng.random(N).astype(np.float32)
        p_lut = rng.random(B).astype(np.float32)
        out = A.arrol_prune_bernoulli(torch.from_numpy(s).to(DEV), torch.from_numpy(u).to(DEV),
                                      torch.from_numpy(p_lut).to(DEV), want_p=True)
        torch.cuda.synchronize()
        p_o, keep_o, surv_o, n_o = O.prune_bernoulli(s, u, p_lut)
        want = np.full(N, -1, dtype=np.int32)
        want[:n_o] = surv_o
        tag = (case, N, B)
        assert np.array_equal(npy(out["p"]), p_o), tag
        assert np.array_equal(npy(out["keep_mask"]), keep_o), tag
        assert np.array_equal(npy(out["survivor_idx"]), want) and int(out["n_survivors"]) == n_o, tag
