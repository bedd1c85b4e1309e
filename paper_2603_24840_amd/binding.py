"""Thin ctypes binding over libarrol.so (the C ABI declared in include/arrol.h).

Argument marshalling only: every stage runs in the library's HIP kernels.  torch is used
for device memory and streams.  There is no CPU fallback: if the library is missing or a
tensor is not on the GPU the call raises.
"""
import ctypes
import functools
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libarrol.so")

OK, EINVAL, EWORKSPACE, EHIP = 0, -1, -2, -3
MAX_GROUP = 64


class ArrolError(RuntimeError):
    def __init__(self, fn, code):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (fn, error_string(code), code))


class KVLayout(ctypes.Structure):
    """Geometry of a paged KV pool: [layer][K|V][page][token][kv_head][dim], bf16."""
    _fields_ = [("n_layers", ctypes.c_int32), ("page_tokens", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("n_pages", ctypes.c_int64)]


class Policy(ctypes.Structure):
    """Parameters of the stochastic pruning policy (App. A.4 Eq. 2): keep rate, target ratio, correction
    strength, clip range, Laplace smoothing."""
    _fields_ = [("kappa", ctypes.c_float), ("rho", ctypes.c_float), ("lam", ctypes.c_float),
                ("p_min", ctypes.c_float), ("p_max", ctypes.c_float), ("alpha", ctypes.c_float)]


_lib = None
ABI_VERSION = 200     # arrol_version() of the library whose argument lists _SIGNATURES describes

_vp, _i32, _i64, _f32, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
_SIGNATURES = {
    "arrol_version": (ctypes.c_int, []),
    "arrol_error_string": (ctypes.c_char_p, [ctypes.c_int]),
    "arrol_score": (ctypes.c_int, [_vp, _i64, _vp, _vp, _f32, _i32, _i32, _vp, _vp, _vp]),
    "arrol_score_mlp_workspace_bytes": (_sz, [_i32, _i32, _i32]),
    "arrol_score_mlp": (ctypes.c_int, [_vp, _i64, _vp, _vp, _vp, _vp, _f32, _i32, _i32, _i32, _vp, _vp, _vp, _sz, _vp]),
    "arrol_score_grad_workspace_bytes": (_sz, [_i32, _i32]),
    "arrol_score_grad": (ctypes.c_int, [_vp, _i64, _vp, _vp, _f32, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _sz, _vp]),
    "arrol_score_mlp_grad_workspace_bytes": (_sz, [_i32, _i32, _i32, _i32]),
    "arrol_score_mlp_grad": (ctypes.c_int, [_vp, _i64, _vp, _vp, _vp, _vp, _f32, _vp, _i32, _i32, _i32, _vp, _vp, _vp,
                                            _vp, _vp, _i32, _vp, _sz, _vp]),
    "arrol_adamw_step": (ctypes.c_int, [_vp, _vp, _vp, _vp, _i64, _i32, _f32, _f32, _f32, _f32, _f32, _vp, _vp]),
    "arrol_select": (ctypes.c_int, [_vp, _i32, _i32, _i32, _f32, _vp, _vp, _vp]),
    "arrol_compact_workspace_bytes": (_sz, [_i32]),
    "arrol_compact": (ctypes.c_int, [_vp, KVLayout, _vp, KVLayout, _vp, _vp, _i32, _vp, _i32, _vp, _i32, _i32,
                                     _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "arrol_compact_static": (ctypes.c_int, [_vp, KVLayout, _vp, KVLayout, _vp, _vp, _i32, _vp, _i32, _vp, _i32, _i32,
                                            _vp, _vp, _vp, _vp, _vp, _vp]),
    "arrol_compact_inplace_workspace_bytes": (_sz, [_i64]),
    "arrol_compact_inplace": (ctypes.c_int, [_vp, KVLayout, _vp, _vp, _i32, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp,
                                             _vp, _sz, _vp]),
    "arrol_logprob_workspace_bytes": (_sz, [_i64, _i32, _i32, _i32]),
    "arrol_logprob": (ctypes.c_int, [_vp, _vp, _vp, _i64, _i32, _i32, _vp, _vp, _i32, _vp, _sz, _vp]),
    "arrol_token_confidence_workspace_bytes": (_sz, [_i32, _i32]),
    "arrol_token_confidence": (ctypes.c_int, [_vp, _vp, _vp, _i64, _i32, _i32, _vp, _vp, _sz, _vp]),
    "arrol_trace_confidence_workspace_bytes": (_sz, [_i64, _i32]),
    "arrol_trace_confidence": (ctypes.c_int, [_vp, _vp, _i64, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _sz, _vp]),
    "arrol_grpo_advantage": (ctypes.c_int, [_vp, _vp, _i64, _i32, _i32, _f32, _vp, _vp, _vp]),
    "arrol_grpo_objective_workspace_bytes": (_sz, [_i32]),
    "arrol_grpo_objective": (ctypes.c_int, [_vp, _vp, _vp, _i64, _i32, _vp, _vp, _f32, _f32, _f32, _vp, _vp, _vp,
                                            _vp, _sz, _vp]),
    "arrol_weighted_vote": (ctypes.c_int, [_vp, _vp, _i32, _i32, _i32, _vp, _vp, _vp]),
    "arrol_histogram": (ctypes.c_int, [_vp, _vp, _i64, _i32, _vp, _vp, _vp]),
    "arrol_calibrate": (ctypes.c_int, [_vp, _vp, _i32, Policy, _vp, _vp, _vp, _vp]),
    "arrol_prune_bernoulli": (ctypes.c_int, [_vp, _vp, _i32, _vp, _i32, _vp, _vp, _vp, _vp, _vp]),
    "arrol_probe_mfma_rate": (ctypes.c_int, [_vp, _i64, _vp, _i64, _i32, _i32, _i32, _vp, _vp, _vp]),
}


def lib():
    """Loads libarrol.so once; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libarrol.so is not built (%s missing): run "
                               "`python -m paper_2603_24840_amd.build`; there is no fallback path" % LIB_PATH)
        handle = ctypes.CDLL(LIB_PATH)
        missing = [name for name in _SIGNATURES if not hasattr(handle, name)]
        handle.arrol_version.restype, handle.arrol_version.argtypes = _SIGNATURES["arrol_version"]
        if missing or handle.arrol_version() != ABI_VERSION:
            raise RuntimeError("%s is a stale build (version %d, this binding is written for %d%s): rebuild with "
                               "`python -m paper_2603_24840_amd.build`" % (LIB_PATH, handle.arrol_version(), ABI_VERSION,
                                                                          "; missing " + ", ".join(missing) if missing else ""))
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def version():
    return lib().arrol_version()


def error_string(code):
    return lib().arrol_error_string(code).decode()


def _ptr(t, dtype=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU: the ARRoL path has no CPU implementation" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return t.data_ptr()


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def _check(fn, rc):
    if rc != OK:
        raise ArrolError(fn, rc)


def _on_stream(fn):
    """Runs the wrapped call with `stream` (when given) as torch's current stream, so that every tensor the
    binding creates itself - outputs and temporary workspaces - belongs to the stream the kernels are
    enqueued on: the caching allocator then cannot hand a dropped temporary to other work while a kernel
    of that stream still uses it."""
    @functools.wraps(fn)
    def wrapper(*args, stream=None, **kwargs):
        if stream is None:
            return fn(*args, stream=None, **kwargs)
        with torch.cuda.stream(stream):
            return fn(*args, stream=stream, **kwargs)
    return wrapper


@_on_stream
def arrol_score(hidden, w, bias=0.0, row_index=None, out_score=None, out_prob=None, want_score=True,
                stream=None):
    """hidden bf16 [R, d] (rows may be strided), w fp32 [d] -> (score fp32 [n], prob fp32 [n])."""
    if hidden.dim() != 2 or hidden.dtype != torch.bfloat16 or not hidden.is_cuda:
        raise TypeError("hidden must be a 2-D bf16 GPU tensor")
    if hidden.stride(1) != 1:
        raise ValueError("hidden rows must be contiguous")
    d = hidden.shape[1]
    n = hidden.shape[0] if row_index is None else row_index.numel()
    dev = hidden.device
    if out_score is None and want_score:
        out_score = torch.empty(n, dtype=torch.float32, device=dev)
    if out_prob is None:
        out_prob = torch.empty(n, dtype=torch.float32, device=dev)
    row_stride = hidden.stride(0) if hidden.shape[0] > 1 else max(d, hidden.stride(0))
    rc = lib().arrol_score(hidden.data_ptr(), row_stride, _ptr(row_index, torch.int64, "row_index"),
                           _ptr(w, torch.float32, "w"), float(bias), n, d,
                           _ptr(out_score, torch.float32, "out_score"), _ptr(out_prob, torch.float32, "out_prob"),
                           _stream(stream))
    _check("arrol_score", rc)
    return out_score, out_prob


@_on_stream
def arrol_score_mlp(hidden, w1, b1, w2, b2=0.0, row_index=None, workspace="auto", stream=None):
    """hidden bf16 [R, d], w1 bf16 [m, d], b1 fp32 [m] or None, w2 fp32 [m] -> (score, prob) fp32 [n].
    workspace: "auto" allocates what the library asks for (the small-batch path), None passes none (the
    one-launch kernel), or a uint8 tensor."""
    if hidden.dim() != 2 or hidden.dtype != torch.bfloat16 or not hidden.is_cuda or hidden.stride(1) != 1:
        raise TypeError("hidden must be a 2-D bf16 GPU tensor with contiguous rows")
    d = hidden.shape[1]
    m = w1.shape[0]
    if w1.shape[1] != d or w2.numel() != m or (b1 is not None and b1.numel() != m):
        raise ValueError("w1 must be [m, d], b1 and w2 [m]")
    n = hidden.shape[0] if row_index is None else row_index.numel()
    dev = hidden.device
    score = torch.empty(n, dtype=torch.float32, device=dev)
    prob = torch.empty(n, dtype=torch.float32, device=dev)
    if isinstance(workspace, str):
        need = lib().arrol_score_mlp_workspace_bytes(n, d, m)
        workspace = torch.empty(need, dtype=torch.uint8, device=dev) if need else None
    row_stride = hidden.stride(0) if hidden.shape[0] > 1 else max(d, hidden.stride(0))
    rc = lib().arrol_score_mlp(hidden.data_ptr(), row_stride, _ptr(row_index, torch.int64, "row_index"),
                               _ptr(w1, torch.bfloat16, "w1"), _ptr(b1, torch.float32, "b1"),
                               _ptr(w2, torch.float32, "w2"), float(b2), n, d, m, score.data_ptr(), prob.data_ptr(),
                               _ptr(workspace, torch.uint8, "workspace"), workspace.numel() if workspace is not None else 0,
                               _stream(stream))
    _check("arrol_score_mlp", rc)
    return score, prob


@_on_stream
def arrol_score_grad(hidden, w, bias, labels, row_index=None, workspace=None, stream=None):
    """Cross-entropy loss of the linear head and its gradient: hidden bf16 [R, d], w fp32 [d], labels fp32 [n]
    -> (loss fp32 [1], grad_w fp32 [d], grad_bias fp32 [1])."""
    if hidden.dim() != 2 or hidden.dtype != torch.bfloat16 or not hidden.is_cuda or hidden.stride(1) != 1:
        raise TypeError("hidden must be a 2-D bf16 GPU tensor with contiguous rows")
    d = hidden.shape[1]
    n = hidden.shape[0] if row_index is None else row_index.numel()
    if labels.numel() != n or w.numel() != d:
        raise ValueError("labels must be [n] and w [d]")
    dev = hidden.device
    need = lib().arrol_score_grad_workspace_bytes(n, d)
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=dev)
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    grad_w = torch.empty(d, dtype=torch.float32, device=dev)
    grad_b = torch.empty(1, dtype=torch.float32, device=dev)
    row_stride = hidden.stride(0) if hidden.shape[0] > 1 else max(d, hidden.stride(0))
    rc = lib().arrol_score_grad(hidden.data_ptr(), row_stride, _ptr(row_index, torch.int64, "row_index"),
                                _ptr(w, torch.float32, "w"), float(bias), _ptr(labels, torch.float32, "labels"), n, d,
                                loss.data_ptr(), grad_w.data_ptr(), grad_b.data_ptr(),
                                _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream))
    _check("arrol_score_grad", rc)
    return loss, grad_w, grad_b


@_on_stream
def arrol_score_mlp_grad(hidden, w1, b1, w2, b2, labels, row_index=None, delta_terms=1, workspace=None, stream=None):
    """Cross-entropy loss of the MLP head and its gradients: -> dict(loss [1], grad_w1 [m, d], grad_b1 [m],
    grad_w2 [m], grad_b2 [1]), all fp32.  delta_terms=2: dL/dW1 to fp32 accuracy (two bf16 terms per delta)."""
    if hidden.dim() != 2 or hidden.dtype != torch.bfloat16 or not hidden.is_cuda or hidden.stride(1) != 1:
        raise TypeError("hidden must be a 2-D bf16 GPU tensor with contiguous rows")
    d = hidden.shape[1]
    m = w1.shape[0]
    n = hidden.shape[0] if row_index is None else row_index.numel()
    if w1.shape[1] != d or w2.numel() != m or (b1 is not None and b1.numel() != m) or labels.numel() != n:
        raise ValueError("w1 must be [m, d], b1 and w2 [m], labels [n]")
    dev = hidden.device
    if workspace is None:
        workspace = torch.empty(max(lib().arrol_score_mlp_grad_workspace_bytes(n, d, m, int(delta_terms)), 256), dtype=torch.uint8,
                                device=dev)
    out = dict(loss=torch.empty(1, dtype=torch.float32, device=dev),
               grad_w1=torch.empty((m, d), dtype=torch.float32, device=dev),
               grad_b1=torch.empty(m, dtype=torch.float32, device=dev),
               grad_w2=torch.empty(m, dtype=torch.float32, device=dev),
               grad_b2=torch.empty(1, dtype=torch.float32, device=dev))
    row_stride = hidden.stride(0) if hidden.shape[0] > 1 else max(d, hidden.stride(0))
    rc = lib().arrol_score_mlp_grad(hidden.data_ptr(), row_stride, _ptr(row_index, torch.int64, "row_index"),
                                    _ptr(w1, torch.bfloat16, "w1"), _ptr(b1, torch.float32, "b1"),
                                    _ptr(w2, torch.float32, "w2"), float(b2), _ptr(labels, torch.float32, "labels"),
                                    n, d, m, out["loss"].data_ptr(), out["grad_w1"].data_ptr(),
                                    out["grad_b1"].data_ptr(), out["grad_w2"].data_ptr(), out["grad_b2"].data_ptr(),
                                    int(delta_terms), _ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
                                    _stream(stream))
    _check("arrol_score_mlp_grad", rc)
    return out


@_on_stream
def arrol_adamw_step(param, grad, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0,
                     param_bf16=None, stream=None):
    """In-place AdamW update of fp32 param / m / v (all [n]); param_bf16 (optional, bf16 [n]) gets a rounded copy."""
    n = param.numel()
    if grad.numel() != n or m.numel() != n or v.numel() != n or (param_bf16 is not None and param_bf16.numel() != n):
        raise ValueError("param, grad, m, v (and param_bf16) must have the same number of elements")
    rc = lib().arrol_adamw_step(_ptr(param, torch.float32, "param"), _ptr(grad, torch.float32, "grad"),
                                _ptr(m, torch.float32, "m"), _ptr(v, torch.float32, "v"), n, int(step), float(lr),
                                float(beta1), float(beta2), float(eps), float(weight_decay),
                                _ptr(param_bf16, torch.bfloat16, "param_bf16"), _stream(stream))
    _check("arrol_adamw_step", rc)
    return param


@_on_stream
def arrol_select(prob, n_groups, G, K, rho=0.5, out_keep=None, out_survivors=None, stream=None):
    """prob fp32 [n_groups*G] -> (keep_mask uint8 [n_groups*G], survivor_idx int32 [n_groups*K])."""
    dev = prob.device
    if prob.numel() != n_groups * G:
        raise ValueError("prob must have n_groups*G entries")
    if out_keep is None:
        out_keep = torch.empty(n_groups * G, dtype=torch.uint8, device=dev)
    if out_survivors is None:
        out_survivors = torch.empty(max(0, n_groups * K), dtype=torch.int32, device=dev)
    rc = lib().arrol_select(_ptr(prob, torch.float32, "prob"), n_groups, G, K, float(rho),
                            _ptr(out_keep, torch.uint8, "keep_mask"), _ptr(out_survivors, torch.int32, "survivor_idx"),
                            _stream(stream))
    _check("arrol_select", rc)
    return out_keep, out_survivors


def kv_layout_of(kv):
    """KVLayout of a [L, 2, P, page_tokens, H_kv, hd] bf16 tensor."""
    if kv.dim() != 6 or kv.shape[1] != 2:
        raise ValueError("KV pool must be [layers, 2, pages, page_tokens, kv_heads, head_dim]")
    L, _, P, pt, H, hd = kv.shape
    return KVLayout(L, pt, H, hd, P)


def arrol_compact_workspace_bytes(n_keep):
    return lib().arrol_compact_workspace_bytes(n_keep)


@_on_stream
def arrol_compact(kv_src, kv_dst, block_table_src, seq_len_src, tokens_src, survivor_idx,
                  out=None, workspace=None, stream=None):
    """Gathers survivors into kv_dst (written in place).  Returns a dict with block_table_dst,
    seq_len_dst, tokens_dst, src_of_dst, n_pages_used (device int64 scalar tensor)."""
    dev = kv_src.device
    n_src, ppr = block_table_src.shape
    n_keep = survivor_idx.numel()
    max_len = tokens_src.shape[1] if tokens_src is not None else 0
    if out is None:
        out = dict(
            block_table_dst=torch.empty((n_keep, ppr), dtype=torch.int32, device=dev),
            seq_len_dst=torch.empty(n_keep, dtype=torch.int32, device=dev),
            tokens_dst=(torch.empty((n_keep, max_len), dtype=torch.int32, device=dev)
                        if tokens_src is not None else None),
            src_of_dst=torch.empty(n_keep, dtype=torch.int32, device=dev),
            n_pages_used=torch.empty(1, dtype=torch.int64, device=dev))
    need = arrol_compact_workspace_bytes(n_keep)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    rc = lib().arrol_compact(
        _ptr(kv_src, torch.bfloat16, "kv_src"), kv_layout_of(kv_src),
        _ptr(kv_dst, torch.bfloat16, "kv_dst"), kv_layout_of(kv_dst),
        _ptr(block_table_src, torch.int32, "block_table_src"), _ptr(seq_len_src, torch.int32, "seq_len_src"),
        ppr, _ptr(tokens_src, torch.int32, "tokens_src"), max_len,
        _ptr(survivor_idx, torch.int32, "survivor_idx"), n_src, n_keep,
        _ptr(out["block_table_dst"], torch.int32, "block_table_dst"), _ptr(out["seq_len_dst"], torch.int32, "seq_len_dst"),
        _ptr(out["tokens_dst"], torch.int32, "tokens_dst"), _ptr(out["src_of_dst"], torch.int32, "src_of_dst"),
        _ptr(out["n_pages_used"], torch.int64, "n_pages_used"),
        _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream))
    _check("arrol_compact", rc)
    return out


@_on_stream
def arrol_compact_static(kv_src, kv_dst, block_table_src, seq_len_src, tokens_src, survivor_idx, out, stream=None):
    """arrol_compact without a workspace: the library's fixed scratch array is used and nothing is allocated
    (every output tensor is the caller's: `out` as returned by arrol_compact)."""
    n_src, ppr = block_table_src.shape
    n_keep = survivor_idx.numel()
    max_len = tokens_src.shape[1] if tokens_src is not None else 0
    rc = lib().arrol_compact_static(
        _ptr(kv_src, torch.bfloat16, "kv_src"), kv_layout_of(kv_src),
        _ptr(kv_dst, torch.bfloat16, "kv_dst"), kv_layout_of(kv_dst),
        _ptr(block_table_src, torch.int32, "block_table_src"), _ptr(seq_len_src, torch.int32, "seq_len_src"),
        ppr, _ptr(tokens_src, torch.int32, "tokens_src"), max_len,
        _ptr(survivor_idx, torch.int32, "survivor_idx"), n_src, n_keep,
        _ptr(out["block_table_dst"], torch.int32, "block_table_dst"), _ptr(out["seq_len_dst"], torch.int32, "seq_len_dst"),
        _ptr(out["tokens_dst"], torch.int32, "tokens_dst"), _ptr(out["src_of_dst"], torch.int32, "src_of_dst"),
        _ptr(out["n_pages_used"], torch.int64, "n_pages_used"), _stream(stream))
    _check("arrol_compact_static", rc)
    return out


@_on_stream
def arrol_compact_inplace(kv, block_table_src, seq_len_src, survivor_idx, workspace=None, stream=None):
    """Moves the survivors' pages into the dense prefix of the SAME pool (kv is modified in place).
    Returns dict(block_table_dst, seq_len_dst, src_of_dst, n_pages_used, n_moved)."""
    dev = kv.device
    n_src, ppr = block_table_src.shape
    n_keep = survivor_idx.numel()
    out = dict(block_table_dst=torch.empty((n_keep, ppr), dtype=torch.int32, device=dev),
               seq_len_dst=torch.empty(n_keep, dtype=torch.int32, device=dev),
               src_of_dst=torch.empty(n_keep, dtype=torch.int32, device=dev),
               n_pages_used=torch.empty(1, dtype=torch.int64, device=dev),
               n_moved=torch.empty(1, dtype=torch.int64, device=dev))
    lay = kv_layout_of(kv)
    need = lib().arrol_compact_inplace_workspace_bytes(lay.n_pages)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    rc = lib().arrol_compact_inplace(
        _ptr(kv, torch.bfloat16, "kv"), lay, _ptr(block_table_src, torch.int32, "block_table_src"),
        _ptr(seq_len_src, torch.int32, "seq_len_src"), ppr, _ptr(survivor_idx, torch.int32, "survivor_idx"),
        n_src, n_keep, out["block_table_dst"].data_ptr(), out["seq_len_dst"].data_ptr(),
        out["src_of_dst"].data_ptr(), out["n_pages_used"].data_ptr(), out["n_moved"].data_ptr(),
        _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream))
    _check("arrol_compact_inplace", rc)
    return out


def arrol_logprob_workspace_bytes(T, V, d, n_splits=0):
    return lib().arrol_logprob_workspace_bytes(T, V, d, n_splits)


@_on_stream
def arrol_logprob(hidden, lm_head, targets, out_logprob=None, out_lse=None, want_lse=False,
                  n_splits=0, workspace=None, stream=None):
    """hidden bf16 [T, d], lm_head bf16 [V, d], targets int32 [T] -> logprob fp32 [T] (and lse).
    n_splits = number of vocabulary ranges (0: the library chooses)."""
    T, d = hidden.shape
    V = lm_head.shape[0]
    if lm_head.shape[1] != d:
        raise ValueError("hidden and lm_head disagree on d")
    dev = hidden.device
    if out_logprob is None:
        out_logprob = torch.empty(T, dtype=torch.float32, device=dev)
    if out_lse is None and want_lse:
        out_lse = torch.empty(T, dtype=torch.float32, device=dev)
    need = arrol_logprob_workspace_bytes(T, V, d, n_splits)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    rc = lib().arrol_logprob(_ptr(hidden, torch.bfloat16, "hidden"), _ptr(lm_head, torch.bfloat16, "lm_head"),
                             _ptr(targets, torch.int32, "targets"), T, V, d,
                             _ptr(out_logprob, torch.float32, "logprob_out"), _ptr(out_lse, torch.float32, "lse_out"),
                             int(n_splits), _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream))
    _check("arrol_logprob", rc)
    return (out_logprob, out_lse) if (want_lse or out_lse is not None) else out_logprob


@_on_stream
def arrol_token_confidence(hidden, lm_head, lse, workspace=None, stream=None):
    """hidden bf16 [T, d], lm_head bf16 [V, d], lse fp32 [T] (from arrol_logprob) -> token confidence fp32 [T]."""
    if hidden.dim() != 2 or lm_head.dim() != 2 or hidden.shape[1] != lm_head.shape[1]:
        raise ValueError("hidden must be [T, d] and lm_head [V, d]")
    T, d = hidden.shape
    V = lm_head.shape[0]
    if lse.numel() != T:
        raise ValueError("lse must be [T]")
    dev = hidden.device
    if workspace is None:
        workspace = torch.empty(max(lib().arrol_token_confidence_workspace_bytes(V, d), 16), dtype=torch.uint8, device=dev)
    conf = torch.empty(T, dtype=torch.float32, device=dev)
    rc = lib().arrol_token_confidence(_ptr(hidden, torch.bfloat16, "hidden"), _ptr(lm_head, torch.bfloat16, "lm_head"),
                                      _ptr(lse, torch.float32, "lse"), T, V, d, conf.data_ptr(),
                                      _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream))
    _check("arrol_token_confidence", rc)
    return conf


@_on_stream
def arrol_trace_confidence(conf, cu_seqlens, window, bottom_percent=10, workspace=None, stream=None):
    """conf fp32 [T], cu_seqlens int64 [n+1] -> (trace mean, min window mean, bottom-share window mean) fp64 [n]."""
    T = conf.numel()
    n = cu_seqlens.numel() - 1
    if n < 0:
        raise ValueError("cu_seqlens must hold at least one offset")
    dev = conf.device
    if workspace is None:
        workspace = torch.empty(max(lib().arrol_trace_confidence_workspace_bytes(T, n), 16), dtype=torch.uint8, device=dev)
    outs = [torch.empty(n, dtype=torch.float64, device=dev) for _ in range(3)]
    rc = lib().arrol_trace_confidence(_ptr(conf, torch.float32, "conf"), _ptr(cu_seqlens, torch.int64, "cu_seqlens"),
                                      T, n, int(window), int(bottom_percent), outs[0].data_ptr(), outs[1].data_ptr(),
                                      outs[2].data_ptr(), _ptr(workspace, torch.uint8, "workspace"),
                                      workspace.numel(), _stream(stream))
    _check("arrol_trace_confidence", rc)
    return tuple(outs)


@_on_stream
def arrol_grpo_advantage(reward, group_offsets, ddof=0, eps=0.0, stream=None):
    """reward fp32 [N], group_offsets int64 [n_groups+1] -> (advantage fp32 [N], seq_weight fp32 [N])."""
    N = reward.numel()
    n_groups = group_offsets.numel() - 1
    adv = torch.zeros(N, dtype=torch.float32, device=reward.device)
    wgt = torch.zeros(N, dtype=torch.float32, device=reward.device)
    rc = lib().arrol_grpo_advantage(_ptr(reward, torch.float32, "reward"), _ptr(group_offsets, torch.int64, "group_offsets"),
                                    N, n_groups, int(ddof), float(eps), adv.data_ptr(), wgt.data_ptr(), _stream(stream))
    _check("arrol_grpo_advantage", rc)
    return adv, wgt


@_on_stream
def arrol_grpo_objective(logp, logp_ref, cu_seqlens, advantage, seq_weight, eps_low=0.2, eps_high=0.2, beta=0.0,
                         want_grad=True, workspace=None, stream=None):
    """-> (J fp64 [1], dJ/dlogp fp32 [T] or None, n_clipped int64 [1])."""
    T = logp.numel()
    n = cu_seqlens.numel() - 1
    if logp_ref.numel() != T or advantage.numel() != n or seq_weight.numel() != n:
        raise ValueError("logp/logp_ref must be [T]; advantage/seq_weight [n_seq]")
    dev = logp.device
    if workspace is None:
        workspace = torch.empty(max(lib().arrol_grpo_objective_workspace_bytes(n), 16), dtype=torch.uint8, device=dev)
    J = torch.empty(1, dtype=torch.float64, device=dev)
    grad = torch.empty(T, dtype=torch.float32, device=dev) if want_grad else None
    n_clip = torch.empty(1, dtype=torch.int64, device=dev)
    rc = lib().arrol_grpo_objective(_ptr(logp, torch.float32, "logp"), _ptr(logp_ref, torch.float32, "logp_ref"),
                                    _ptr(cu_seqlens, torch.int64, "cu_seqlens"), T, n,
                                    _ptr(advantage, torch.float32, "advantage"), _ptr(seq_weight, torch.float32, "seq_weight"),
                                    float(eps_low), float(eps_high), float(beta), J.data_ptr(),
                                    None if grad is None else grad.data_ptr(), n_clip.data_ptr(),
                                    _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream))
    _check("arrol_grpo_objective", rc)
    return J, grad, n_clip


@_on_stream
def arrol_weighted_vote(prob, answer_id, n_questions, C, n_answers, want_tally=False, out_winner=None, stream=None):
    """prob fp32 [Q*C], answer_id int32 [Q*C] -> winner int32 [Q] (and tally int64 [Q, A])."""
    dev = prob.device
    if prob.numel() != n_questions * C or answer_id.numel() != n_questions * C:
        raise ValueError("prob and answer_id must have n_questions*C entries")
    winner = out_winner if out_winner is not None else torch.empty(n_questions, dtype=torch.int32, device=dev)
    if winner.numel() != n_questions:
        raise ValueError("out_winner must have n_questions entries")
    tally = torch.empty((n_questions, n_answers), dtype=torch.int64, device=dev) if want_tally else None
    rc = lib().arrol_weighted_vote(_ptr(prob, torch.float32, "prob"), _ptr(answer_id, torch.int32, "answer_id"),
                                   n_questions, C, n_answers, _ptr(winner, torch.int32, "winner"),
                                   _ptr(tally, torch.int64, "tally"), _stream(stream))
    _check("arrol_weighted_vote", rc)
    return (winner, tally) if want_tally else winner


@_on_stream
def arrol_histogram(s_norm, label, B, stream=None):
    """s_norm fp32 [M] in [0,1], label uint8 [M] -> (c_pos, c_neg) int64 [B]."""
    dev = s_norm.device
    c_pos = torch.empty(B, dtype=torch.int64, device=dev)
    c_neg = torch.empty(B, dtype=torch.int64, device=dev)
    rc = lib().arrol_histogram(_ptr(s_norm, torch.float32, "s_norm"), _ptr(label, torch.uint8, "label"),
                               s_norm.numel(), B, c_pos.data_ptr(), c_neg.data_ptr(), _stream(stream))
    _check("arrol_histogram", rc)
    return c_pos, c_neg


@_on_stream
def arrol_calibrate(c_pos, c_neg, policy, stream=None):
    """int64 histograms [B] + Policy -> (q_lut fp32 [B], p_lut fp32 [B], delta fp64 device scalar)."""
    B = c_pos.numel()
    dev = c_pos.device
    q_lut = torch.empty(B, dtype=torch.float32, device=dev)
    p_lut = torch.empty(B, dtype=torch.float32, device=dev)
    delta = torch.empty(1, dtype=torch.float64, device=dev)
    rc = lib().arrol_calibrate(_ptr(c_pos, torch.int64, "c_pos"), _ptr(c_neg, torch.int64, "c_neg"), B, policy,
                               q_lut.data_ptr(), p_lut.data_ptr(), delta.data_ptr(), _stream(stream))
    _check("arrol_calibrate", rc)
    return q_lut, p_lut, delta


@_on_stream
def arrol_prune_bernoulli(s_norm, uniforms, p_lut, want_p=False, stream=None):
    """s_norm, uniforms fp32 [N], p_lut fp32 [B] -> dict(keep_mask, survivor_idx (padded with -1),
    n_survivors (device int32), p (optional))."""
    N = s_norm.numel()
    dev = s_norm.device
    out = dict(keep_mask=torch.empty(N, dtype=torch.uint8, device=dev),
               survivor_idx=torch.empty(N, dtype=torch.int32, device=dev),
               n_survivors=torch.empty(1, dtype=torch.int32, device=dev),
               p=torch.empty(N, dtype=torch.float32, device=dev) if want_p else None)
    rc = lib().arrol_prune_bernoulli(_ptr(s_norm, torch.float32, "s_norm"), _ptr(uniforms, torch.float32, "uniforms"),
                                     N, _ptr(p_lut, torch.float32, "p_lut"), p_lut.numel(),
                                     _ptr(out["p"], torch.float32, "p_out"), out["keep_mask"].data_ptr(),
                                     out["survivor_idx"].data_ptr(), out["n_survivors"].data_ptr(), _stream(stream))
    _check("arrol_prune_bernoulli", rc)
    return out


@_on_stream
def arrol_probe_mfma_rate(a, b, shape=16, n_workgroups=256, iters=1000, out_sink=None, stream=None):
    """Measurement aid: register-only bf16 MFMA loop on the values of a and b (bf16, whole 512-element
    fragments).  Returns (sink fp32 [n_workgroups * 512], flop count of the launch)."""
    sink = out_sink if out_sink is not None else torch.empty(n_workgroups * 512, dtype=torch.float32, device=a.device)
    flop = ctypes.c_double(0.0)
    rc = lib().arrol_probe_mfma_rate(_ptr(a, torch.bfloat16, "a"), a.numel(), _ptr(b, torch.bfloat16, "b"), b.numel(),
                                     shape, n_workgroups, iters, _ptr(sink, torch.float32, "sink"),
                                     ctypes.byref(flop), _stream(stream))
    _check("arrol_probe_mfma_rate", rc)
    return sink, flop.value
