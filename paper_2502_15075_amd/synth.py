"""Seeded synthetic K / V / q tensors shaped like one transformer layer's decode step.

This module only draws random numbers and scales them; it holds none of the method's
arithmetic, so both the GPU library's tests and the CPU oracle's tests may use it.

Recipe (stands in for real model activations, which need weights and datasets):
  K ~ N(0,1) * sigma_k with a few fixed head_dim channels multiplied by `outlier_scale`
  (keys of real models carry a handful of large-magnitude channels and a larger norm than
  values: Sec. 3, Theorem 1 and Fig. "svd"), V ~ N(0,1), q ~ N(0,1).
Draw order from one generator seeded with `seed`: K, V, q, each as float32, then cast.
"""
from __future__ import annotations

import torch

OUTLIER_CHANNELS = (5, 37, 69, 101)


def make_kvq(seed: int, batch: int, kv_heads: int, q_heads: int, seq: int, head_dim: int = 128,
             dtype: torch.dtype = torch.float16, sigma_k: float = 4.0, outlier_scale: float = 20.0,
             outlier_channels=OUTLIER_CHANNELS, device: str = "cpu"):
    """Returns K, V of shape [batch, kv_heads, seq, head_dim] and q of shape [batch, q_heads, head_dim]."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    shape = (batch, kv_heads, seq, head_dim)

    def draw(shp, scale=None):
        # one (batch) slice at a time keeps the float32 temporary small for the large shapes
        out = torch.empty(shp, dtype=dtype, device=device)
        for b in range(shp[0]):
            x = torch.randn(shp[1:], generator=g, dtype=torch.float32, device=device)
            if scale is not None:
                x = scale(x)
            out[b] = x.to(dtype)
        return out

    def kscale(x):
        x = x * sigma_k
        if outlier_scale != 1.0 and len(outlier_channels):
            x[..., list(outlier_channels)] *= outlier_scale
        return x

    K = draw(shape, kscale)
    V = draw(shape)
    q = draw((batch, q_heads, head_dim))
    return K, V, q


def to_numpy_bits(t: torch.Tensor):
    """Host numpy view for the oracle: float16 -> float16 array, bfloat16 -> uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        import numpy as np
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
