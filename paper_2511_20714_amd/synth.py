"""Seeded synthetic inputs shaped like Wan-class DiT self-attention under
block diffusion.  Input generation only: none of the attention or cache
arithmetic lives here, and both the HIP tests and the CPU oracle's tests draw
from this one module.

Recipe: q, k, v ~ iid N(0, 1) per element from a generator keyed by
(seed, block, step, layer); with ``rms_norm`` every (token, head) row of q and k
is divided by sqrt(mean(x^2) + 1e-6) in fp32 (QK-normed DiT, no gain, no RoPE);
``logit_gain`` multiplies q (a "peaked" variant with a few dominant keys);
finally the values are rounded to the storage dtype.
"""
from __future__ import annotations

import torch


def _key(seed: int, block: int, step: int, layer: int) -> int:
    x = (seed * 0x9E3779B97F4A7C15 + block * 0xBF58476D1CE4E5B9 + step * 0x94D049BB133111EB + layer * 0xD6E8FEB86659FD93)
    return x % (1 << 62)


def draw_qkv(seed, block, step, layer, n, heads, head_dim, dtype, device, rms_norm=False, logit_gain=1.0):
    """Returns (q, k, v), each [n, heads, head_dim] of ``dtype`` on ``device``."""
    g = torch.Generator(device=device)
    g.manual_seed(_key(seed, block, step, layer))
    x = torch.randn((3, n, heads, head_dim), generator=g, device=device, dtype=torch.float32)
    q, k, v = x[0], x[1], x[2]
    if rms_norm:
        q = q / torch.sqrt(q.pow(2).mean(-1, keepdim=True) + 1e-6)
        k = k / torch.sqrt(k.pow(2).mean(-1, keepdim=True) + 1e-6)
    if logit_gain != 1.0:
        q = q * logit_gain
    return q.to(dtype).contiguous(), k.to(dtype).contiguous(), v.to(dtype).contiguous()


def to_f64_numpy(t: torch.Tensor):
    """Exact widening of a (possibly device, possibly bf16) tensor to a float64 numpy array."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def raw_bytes(t: torch.Tensor) -> bytes:
    """The tensor's storage bytes (for bit-exact comparisons)."""
    t = t.detach().to("cpu").contiguous()
    if t.dtype == torch.bfloat16:
        t = t.view(torch.int16)
    return t.numpy().tobytes()
