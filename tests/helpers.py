"""Test-side glue: move torch tensors to the numpy forms the oracle takes."""
import numpy as np
import torch

from paper_2603_24840_amd.workloads import bits, npy  # noqa: F401  (host views shared with bench.py and smoke())


def f32_to_bf16_bits(x):
    """Round-to-nearest-even float32 -> bf16 bit patterns."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def bf16_tensor_from_bits(b, device):
    return torch.from_numpy(np.ascontiguousarray(b).view(np.int16)).view(torch.bfloat16).to(device)


def to_dev(x, device, dtype=None):
    """numpy array (an input, or an oracle result rounded to the interface dtype) -> device tensor."""
    a = np.ascontiguousarray(x if dtype is None else np.asarray(x).astype(dtype))
    return torch.from_numpy(a).to(device)


def oracle_survivors(O, prob_f32, cfg):
    """Survivors the oracle selects from fp32 probabilities (numpy), as (keep_mask, survivor_idx)."""
    return O.select(np.asarray(prob_f32, dtype=np.float32), cfg.n_prompts, cfg.G, cfg.K, cfg.rho)
