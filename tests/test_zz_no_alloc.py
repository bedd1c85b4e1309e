"""arrol_compact_static (the entry point that allocates nothing) against arrol_compact, through the C ABI:
two calls in a row on the same GPU, the second with a smaller input, every output compared bit for bit."""
import ctypes

import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _outputs(n_keep, ppr, max_len):
    return dict(block_table_dst=torch.full((n_keep, ppr), -7, dtype=torch.int32, device=DEV),
                seq_len_dst=torch.full((n_keep,), -7, dtype=torch.int32, device=DEV),
                tokens_dst=torch.full((n_keep, max_len), -7, dtype=torch.int32, device=DEV),
                src_of_dst=torch.full((n_keep,), -7, dtype=torch.int32, device=DEV),
                n_pages_used=torch.full((1,), -7, dtype=torch.int64, device=DEV))


def _case(A, W, n_prompts, seed):
    """Seeded ragged batch with the tiny configuration's geometry; survivors chosen by a seeded draw."""
    cfg = W.shrink(W.CONFIGS["tiny"], n_prompts=n_prompts)
    kv, bt, sl, tok = W.compact_inputs(cfg, DEV, extra_pages=5, ragged=True)
    g = torch.Generator(device="cpu"); g.manual_seed(seed)
    surv = torch.sort(torch.randperm(cfg.n_rollouts, generator=g)[:cfg.n_keep])[0].to(torch.int32).to(DEV)
    return cfg, kv, bt, sl, tok, surv


def _run_both(A, cfg, kv, bt, sl, tok, surv):
    L = A.lib()
    n_src, ppr = bt.shape
    n_keep, max_len = surv.numel(), tok.shape[1]
    n_dst = n_keep * ppr
    lay_s = A.kv_layout_of(kv)
    results = []
    for static in (False, True):
        dst = torch.empty((cfg.n_layers, 2, n_dst) + tuple(kv.shape[3:]), dtype=torch.bfloat16, device=DEV)
        dst.view(torch.int16).fill_(0x7FC1)
        out = _outputs(n_keep, ppr, max_len)
        lay_d = A.kv_layout_of(dst)
        common = (_ptr(kv), lay_s, _ptr(dst), lay_d, _ptr(bt), _ptr(sl), ppr, _ptr(tok), max_len, _ptr(surv),
                  n_src, n_keep, _ptr(out["block_table_dst"]), _ptr(out["seq_len_dst"]), _ptr(out["tokens_dst"]),
                  _ptr(out["src_of_dst"]), _ptr(out["n_pages_used"]))
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        if static:
            rc = L.arrol_compact_static(*common, stream)
        else:
            ws = torch.empty(max(16, L.arrol_compact_workspace_bytes(n_keep)), dtype=torch.uint8, device=DEV)
            rc = L.arrol_compact(*common, _ptr(ws), ws.numel(), stream)
        assert rc == 0, rc
        torch.cuda.synchronize()
        results.append((dst, out))
    (dst_a, out_a), (dst_b, out_b) = results
    assert torch.equal(dst_a.view(torch.int16), dst_b.view(torch.int16))
    for k in out_a:
        assert torch.equal(out_a[k], out_b[k]), k
    assert int(out_b["n_pages_used"][0]) > 0


def test_compact_static_matches_compact_on_two_calls_in_a_row():
    import paper_2603_24840_amd as A
    from paper_2603_24840_amd import workloads as W
    A.lib()
    print("[case] arrol_compact_static vs arrol_compact: 24 prompts then 5 prompts", flush=True)
    _run_both(A, *_case(A, W, 24, seed=1))     # 96 survivors
    _run_both(A, *_case(A, W, 5, seed=2))      # 20 survivors: the scratch still holds the larger call's offsets
