"""Parity of the in-place (hole-filling) KV compaction with the oracle: bit-exact pool, tables and counts."""
import numpy as np
import pytest
import torch

import oracle as O
from helpers import bits, npy, to_dev, oracle_survivors

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


def run_case(A, kv, bt, sl, surv):
    ref_kv = bits(kv).copy()
    ref = O.compact_inplace(ref_kv, npy(bt), npy(sl), npy(surv))
    out = A.arrol_compact_inplace(kv, bt, sl, surv)
    torch.cuda.synchronize()
    assert int(out["n_pages_used"][0]) == ref["n_pages_used"] and int(out["n_moved"][0]) == ref["n_moved"]
    assert np.array_equal(npy(out["block_table_dst"]), ref["block_table_dst"])
    assert np.array_equal(npy(out["seq_len_dst"]), ref["seq_len_dst"])
    assert np.array_equal(npy(out["src_of_dst"]), ref["src_of_dst"])
    assert np.array_equal(bits(kv), ref_kv)                      # the whole pool, moved and untouched pages alike
    return out, ref


def test_inplace_tiny_config(A, W):
    cfg = W.CONFIGS["tiny"]
    print("[case] inplace tiny", flush=True)
    kv, bt, sl, _ = W.compact_inputs(cfg, DEV)
    _, surv_o = oracle_survivors(O, npy(W.select_inputs(cfg, DEV)), cfg)      # survivors from the oracle's selection
    surv = to_dev(surv_o, DEV)
    out, ref = run_case(A, kv, bt, sl, surv)
    assert ref["n_pages_used"] == cfg.n_keep * cfg.pages_per_rollout and 0 < ref["n_moved"] < ref["n_pages_used"]


@pytest.mark.parametrize("head_dim,pt,n_prompts,G,K,extra", [(64, 16, 6, 5, 2, 5), (128, 16, 40, 8, 4, 0), (8, 1, 3, 4, 1, 3),
                                                          (40, 3, 9, 3, 3, 1), (64, 16, 300, 8, 4, 77)])
def test_inplace_ragged(A, W, head_dim, pt, n_prompts, G, K, extra):
    print("[case] inplace hd=%d page=%d prompts=%d G=%d K=%d" % (head_dim, pt, n_prompts, G, K), flush=True)
    cfg = W.shrink(W.CONFIGS["tiny"], n_prompts=n_prompts, G=G, K=K, head_dim=head_dim, page_tokens=pt, ckpt_len=37,
                   n_layers=2, n_kv_heads=2)
    kv, bt, sl, _ = W.compact_inputs(cfg, DEV, extra_pages=extra, ragged=True)
    g = torch.Generator(device="cpu"); g.manual_seed(n_prompts)
    pick = torch.stack([torch.sort(torch.randperm(G, generator=g)[:K])[0] + i * G
                        for i in range(n_prompts)]).reshape(-1).to(torch.int32).to(DEV)
    run_case(A, kv, bt, sl, pick)


@pytest.mark.parametrize("n_prompts,G,K,extra,pt", [(5, 6, 3, 3, 16), (300, 8, 4, 77, 16), (1, 2, 1, 0, 16), (40, 4, 2, 9, 32)])
def test_inplace_chunks_of_32_kib_and_more(A, W, n_prompts, G, K, extra, pt):
    """head_dim 128 x 8 KV heads x 16 tokens = 32 KiB per chunk (64 KiB with 32-token pages): the copy runs as a
    persistent grid there - fewer copies than workgroups, and several copies per workgroup."""
    print("[case] inplace 32 KiB chunks prompts=%d G=%d K=%d page=%d" % (n_prompts, G, K, pt), flush=True)
    cfg = W.shrink(W.CONFIGS["tiny"], n_prompts=n_prompts, G=G, K=K, head_dim=128, page_tokens=pt, ckpt_len=37 * pt // 16,
                   n_layers=2, n_kv_heads=8)
    assert cfg.chunk_bytes >= 32768
    kv, bt, sl, _ = W.compact_inputs(cfg, DEV, extra_pages=extra, ragged=True)
    g = torch.Generator(device="cpu"); g.manual_seed(n_prompts)
    pick = torch.stack([torch.sort(torch.randperm(G, generator=g)[:K])[0] + i * G
                        for i in range(n_prompts)]).reshape(-1).to(torch.int32).to(DEV)
    _, ref = run_case(A, kv, bt, sl, pick)
    if n_prompts == 300:
        assert ref["n_moved"] * 4 > 1024      # more copies than the grid has workgroups


def test_inplace_degenerate_cases(A, W):
    cfg = W.CONFIGS["tiny"]
    kv, bt, sl, _ = W.compact_inputs(cfg, DEV)
    before = kv.clone()
    # nobody survives: nothing moves, everything is free
    out, _ = run_case(A, kv, bt, sl, torch.empty(0, dtype=torch.int32, device=DEV))
    assert torch.equal(kv.view(torch.int16), before.view(torch.int16))
    # everybody survives and the pool has no spare pages: already dense, nothing moves
    out, ref = run_case(A, kv, bt, sl, torch.arange(cfg.n_rollouts, dtype=torch.int32, device=DEV))
    assert ref["n_moved"] == 0 and torch.equal(kv.view(torch.int16), before.view(torch.int16))
    # invalid survivor ids and out-of-range table entries are ignored
    bt2 = bt.clone(); bt2[5, 1] = -3; bt2[5, 2] = kv.shape[2] + 9
    surv = torch.tensor([5, -1, 9999, 7], dtype=torch.int32, device=DEV)
    out = A.arrol_compact_inplace(kv, bt2, sl, surv)
    torch.cuda.synchronize()
    assert npy(out["src_of_dst"]).tolist() == [5, -1, -1, 7] and int(out["n_pages_used"][0]) == 6
    row = npy(out["block_table_dst"])[0]
    assert row[1] == -1 and row[2] == -1 and 0 <= row[0] < 6 and 0 <= row[3] < 6


@pytest.mark.parametrize("name", ["llama1b", "qwen8b"])
def test_inplace_full_size(A, W, name):
    """llama1b: 8.6 GB pool of 16 KiB chunks (one workgroup per copy); qwen8b: 155 GB pool of 32 KiB chunks (the
    persistent walk, offsets far beyond 4 GiB).  The oracle runs on the first and the last layer, every layer is
    checked by a fingerprint of every survivor page."""
    import gc
    cfg = W.CONFIGS[name]
    print("[case] inplace %s full pool; oracle on 2 of %d layers, content property on all" % (name, cfg.n_layers), flush=True)
    kv, bt, sl, _ = W.compact_inputs(cfg, DEV)
    _, surv_o = oracle_survivors(O, npy(W.select_inputs(cfg, DEV)), cfg)      # survivors from the oracle's selection
    surv = to_dev(surv_o, DEV)
    flat_old = bt[surv.long()].reshape(-1).long()
    probe = kv[:, :, flat_old, 0, 0, :4].clone()                 # a fingerprint of every survivor page, all layers
    host_before = {layer: bits(kv[layer:layer + 1]).copy() for layer in (0, cfg.n_layers - 1)}
    out = A.arrol_compact_inplace(kv, bt, sl, surv)
    torch.cuda.synchronize()
    n_live = cfg.n_keep * cfg.pages_per_rollout
    assert int(out["n_pages_used"][0]) == n_live
    for layer, ref_kv in host_before.items():
        ref = O.compact_inplace(ref_kv, npy(bt), npy(sl), npy(surv))
        assert np.array_equal(bits(kv[layer:layer + 1]), ref_kv), layer
    assert np.array_equal(npy(out["block_table_dst"]), ref["block_table_dst"]) and int(out["n_moved"][0]) == ref["n_moved"]
    flat_new = out["block_table_dst"].reshape(-1).long()
    assert int(flat_new.max()) == n_live - 1 and torch.unique(flat_new).numel() == n_live
    assert torch.equal(kv[:, :, flat_new, 0, 0, :4].view(torch.int16), probe.view(torch.int16))
    del kv, probe, host_before, ref
    gc.collect()
    torch.cuda.empty_cache()


def test_inplace_pool_beyond_the_one_launch_planner(A, W):
    """More than 524,288 pages: the live-page bitmap no longer fits the planning workgroup's LDS and the call
    falls back to the multi-launch planner (flags in the workspace, single-workgroup scan)."""
    print("[case] inplace, 600,000-page pool of 16-byte chunks", flush=True)
    cfg = W.shrink(W.CONFIGS["tiny"], n_prompts=3000, G=4, K=2, head_dim=8, page_tokens=1, ckpt_len=50, n_layers=1,
                   n_kv_heads=1)
    kv, bt, sl, _ = W.compact_inputs(cfg, DEV, extra_pages=123, ragged=True)
    assert kv.shape[2] > 524288
    g = torch.Generator(device="cpu"); g.manual_seed(5)
    pick = torch.stack([torch.sort(torch.randperm(cfg.G, generator=g)[:cfg.K])[0] + i * cfg.G
                        for i in range(cfg.n_prompts)]).reshape(-1).to(torch.int32).to(DEV)
    run_case(A, kv, bt, sl, pick)
