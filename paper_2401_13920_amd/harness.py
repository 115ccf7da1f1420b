"""Plumbing between the seeded workload generators and device memory (no arithmetic of the
method): uploads hidden states and expert weights, one expert at a time, as bf16/fp32 tensors."""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from . import workloads as wl


def torch_dtype(dtype: str):
    import torch
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def to_device(a: np.ndarray, dtype: str, device="cuda"):
    """float32 host array of storage-representable values -> device tensor of the storage dtype."""
    import torch
    if dtype == "bf16":
        bits = wl.f32_to_bf16_bits(a)
        return torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


def bits_to_device(bits: np.ndarray, out=None, device="cuda"):
    import torch
    t = torch.from_numpy(bits.view(np.int16))
    if out is None:
        return t.to(device).view(torch.bfloat16)
    out.view(torch.int16).copy_(t)
    return out


def to_host_f32(t) -> np.ndarray:
    """Device tensor (bf16 or fp32) -> float32 numpy (exact)."""
    import torch
    return t.detach().to(torch.float32).cpu().numpy()


def upload_weights(c: wl.Config, keep=(), device="cuda", workers: int | None = None, progress=None):
    """Generates every expert's (W_in [h,d], W_out [d,h]) with the seeded generator and copies
    it into two device tensors [E,h,d] and [E,d,h] (bf16).  Host memory holds a few experts at a
    time.  ``keep`` lists expert ids whose float32 host copies are returned for the oracle."""
    import torch
    W_in = torch.empty(c.E, c.h, c.d, dtype=torch.bfloat16, device=device)
    W_out = torch.empty(c.E, c.d, c.h, dtype=torch.bfloat16, device=device)
    kept = {}
    workers = workers or min(16, os.cpu_count() or 1, c.E)
    per_expert_bytes = 2 * c.h * c.d * 6            # fp32 scratch + bf16 bits
    workers = max(1, min(workers, int(24e9 // max(per_expert_bytes, 1))))

    def gen(e):
        return e, wl.expert_weights_bits(c, e)

    with ThreadPoolExecutor(max_workers=workers) as ex:
        for e0 in range(0, c.E, workers):
            for e, (b_in, b_out) in ex.map(gen, range(e0, min(c.E, e0 + workers))):
                bits_to_device(b_in, W_in[e])
                bits_to_device(b_out, W_out[e])
                if e in keep:
                    kept[e] = (wl.bf16_bits_to_f32(b_in), wl.bf16_bits_to_f32(b_out))
            if progress:
                progress(min(c.E, e0 + workers), c.E)
    return W_in, W_out, kept
