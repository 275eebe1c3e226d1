"""Seeded synthetic inputs for the VLA forward path (shared by tests, smoke and bench).

This module only draws random numbers and lays them out; it holds none of the
method's arithmetic and imports neither the oracle nor the HIP binding.

The five workloads stand in for the paper's experiments (random-input stability
run of Section 6.2, the multi-query associative recall task of Section 5.2, the
latency sweep of Section 6.1): the paper's trained model and data generator are
not available, so plain Gaussian / unit-key tensors of the same shapes are used.

All tensors are [B, H, T, d] contiguous.  CPU recipes use numpy's PCG64
(`default_rng(seed)`), drawing q, then k, then v.  The two large bf16 workloads
are drawn on the GPU with torch's generator by the caller (see `device_gaussian`).
"""
from __future__ import annotations

import numpy as np

# name -> shape / dtype / value recipe. "lambda0" is the A_0 = I/lambda0 used with it.
CONFIGS = {
    "tiny": dict(B=1, H=1, T=256, d=16, dtype="f32", std=1.0, seed=0, lambda0=1.0),
    "norm_growth": dict(B=8, H=8, T=1000, d=64, dtype="f32", std=1.0, seed=1, lambda0=0.1),
    "recall": dict(B=64, H=4, T=2048, d=64, dtype="f32", seed=2, lambda0=0.1,
                   n_pairs=(16, 32, 48, 64)),
    "long_context": dict(B=1, H=16, d=64, dtype="bf16", std=1.0, seed=3, lambda0=0.1,
                         T_sweep=(4096, 16384, 43008, 65536, 131072)),
    "large_batch": dict(B=64, H=32, T=8192, d=128, dtype="bf16", std=128 ** -0.5, seed=4,
                        lambda0=0.1),
}


def gaussian_qkv(B, H, T, d, seed, std=1.0, d_v=None):
    """q, k, v ~ i.i.d. N(0, std^2) as float32, drawn in that order from PCG64(seed)."""
    d_v = d if d_v is None else d_v
    rng = np.random.default_rng(seed)
    q = (rng.standard_normal((B, H, T, d)) * std).astype(np.float32)
    k = (rng.standard_normal((B, H, T, d)) * std).astype(np.float32)
    v = (rng.standard_normal((B, H, T, d_v)) * std).astype(np.float32)
    return q, k, v


def recall_task(B, H, T, d, seed, n_pairs=(16, 32, 48, 64)):
    """Synthetic multi-query associative recall on the bare recurrence.

    Per (b, h): n = n_pairs[b % len(n_pairs)] random unit-norm keys with N(0,1)
    values.  Write tokens (k = key_i, v = val_i, q = 0) sit at n sorted random
    positions in [0, T/2); query tokens (k = 0, v = 0, q = key_sigma(j)) at n
    sorted random positions in [T/2, T), sigma a random permutation; every other
    token is all-zero filler.  Returns float32 q, k, v and a dict with
    `n` [B,H], `write_pos`, `query_pos`, `sigma` (lists per head) and `values`.
    """
    rng = np.random.default_rng(seed)
    q = np.zeros((B, H, T, d), np.float32)
    k = np.zeros((B, H, T, d), np.float32)
    v = np.zeros((B, H, T, d), np.float32)
    meta = dict(n=np.zeros((B, H), np.int64), write_pos={}, query_pos={}, sigma={}, values={})
    half = T // 2
    for b in range(B):
        n = int(n_pairs[b % len(n_pairs)])
        for h in range(H):
            keys = rng.standard_normal((n, d))
            keys /= np.linalg.norm(keys, axis=1, keepdims=True)
            vals = rng.standard_normal((n, d))
            wpos = np.sort(rng.choice(half, size=n, replace=False))
            qpos = half + np.sort(rng.choice(T - half, size=n, replace=False))
            sigma = rng.permutation(n)
            k[b, h, wpos] = keys.astype(np.float32)
            v[b, h, wpos] = vals.astype(np.float32)
            q[b, h, qpos] = keys[sigma].astype(np.float32)
            meta["n"][b, h] = n
            meta["write_pos"][(b, h)] = wpos
            meta["query_pos"][(b, h)] = qpos
            meta["sigma"][(b, h)] = sigma
            meta["values"][(b, h)] = v[b, h, wpos].copy()
    return q, k, v, meta


def f32_to_bf16_bits(x):
    """Round float32 -> bfloat16 (round-to-nearest-even); returns the uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    rounded = bits + (np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x):
    """float32 values rounded to the nearest bfloat16, returned as float32."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


def device_gaussian(B, H, T, d, seed, std, torch_dtype, device="cuda", d_v=None):
    """q, k, v ~ N(0, std^2) drawn on `device` with torch's generator seeded by `seed`
    (order q, k, v; drawn in float32, then cast to `torch_dtype`)."""
    import torch

    d_v = d if d_v is None else d_v
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    out = []
    for dd in (d, d, d_v):
        x = torch.empty((B, H, T, dd), dtype=torch_dtype, device=device)
        # draw slab by slab so the float32 staging buffer stays small
        for b in range(B):
            x[b] = (torch.randn((H, T, dd), generator=g, device=device, dtype=torch.float32)
                    * std).to(torch_dtype)
        out.append(x)
    return tuple(out)


def sampled_heads(B, H, every=32):
    """Deterministic sample of flat head indices: first, last and every `every`-th."""
    n = B * H
    idx = sorted(set(list(range(0, n, every)) + [n - 1]))
    return idx
