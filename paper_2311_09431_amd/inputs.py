"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds no attention arithmetic: it only draws Gaussians from a seeded
generator and rounds them to the storage dtype, so that the HIP path and the
CPU oracle consume the same bits.  Activations stand in for real Q/K/V: the
paper's workloads (Sec. 3.1, Table 1) are defined by shapes only, head_dim 128
with 16 or 32 heads, sequence lengths 8k to 786k, N = 2..16 devices.
"""
import torch


def gaussian(shape, seed, dtype=torch.float32, std=1.0, device="cpu"):
    """N(0, std^2) tensor of `shape`, drawn in fp32 from a generator seeded with
    `seed` on `device`, then rounded once to `dtype`.  For a given (device type,
    seed, shape) the bits are reproducible."""
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    x = torch.randn(shape, generator=g, dtype=torch.float32, device=device)
    if std != 1.0:
        x = x * std
    return x.to(dtype)


def qkv(B, H, S, d, seed, dtype=torch.float32, device="cpu", with_dout=False):
    """Unpermuted Q, K, V (and optionally dO) of shape [B, H, S, d], i.i.d. N(0, 1)."""
    n = 4 if with_dout else 3
    return tuple(gaussian((B, H, S, d), seed * 16 + i, dtype, device=device) for i in range(n))


def to_f64(t):
    """Host float64 numpy copy of a tensor (exact for fp32 / bf16 storage)."""
    return t.detach().to("cpu").to(torch.float64).numpy()
