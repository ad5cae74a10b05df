"""Helpers for the GPU parity tests: host arrays <-> device tensors."""
import numpy as np
import torch

import fdd_workloads as W


def to_dev(a, dtype=None):
    """numpy array in storage type (uint16 = bf16 bits) -> cuda tensor."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(a).cuda()


def to_f64(t):
    """cuda tensor -> float64 numpy (exact widening)."""
    return t.detach().to(torch.float64).cpu().numpy()


def storage(x, dtype):
    return W.to_storage(np.asarray(x, dtype=np.float32), dtype)


def rand_attn(rng, N, B, L, Hq, Hkv, D, dtype, std=1.0):
    f = lambda *s: storage(rng.standard_normal(s) * std, dtype)
    return dict(q=f(N, B, Hq, D), prefix_k=f(L, Hkv, D), prefix_v=f(L, Hkv, D),
                block_k=f(N, B, Hkv, D), block_v=f(N, B, Hkv, D))


def print_case(**kw):
    print("[case]", " ".join(f"{k}={v}" for k, v in kw.items()), flush=True)
