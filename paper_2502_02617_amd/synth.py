"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds none of the method's arithmetic: it only draws the data that
the encode / attention path is fed with.  The recipes stand in for the
Llama-3.1-8B key/value cache the paper measured on (8 KV heads, 32 query heads,
head dimension 128): i.i.d. N(0,1) entries, a few "outlier" channels per head
scaled up by a log-normal factor, rounded to bf16 before anyone sees them.

Every function is deterministic in its seed for a given device type.  Tests
always draw on the CPU; the benchmark may draw on the GPU (same recipe, other
random stream) and hands samples of what it drew to the CPU baseline.
"""
import numpy as np
import torch

D = 128
N_OUTLIER = 4
OUTLIER_MU = 2.0
OUTLIER_SIGMA = 0.5


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def gaussian_vectors(n, seed=0, device="cpu"):
    """[n, 128] float32, i.i.d. N(0, 1)."""
    return torch.randn(n, D, generator=_gen(seed, device), device=device, dtype=torch.float32)


def outlier_profile(n_heads, seed):
    """Per head: 4 distinct channel indices and their log-normal scales (CPU, float32)."""
    g = _gen(seed, "cpu")
    scale = torch.ones(n_heads, D, dtype=torch.float32)
    for h in range(n_heads):
        idx = torch.randperm(D, generator=g)[:N_OUTLIER]
        s = torch.exp(OUTLIER_MU + OUTLIER_SIGMA * torch.randn(N_OUTLIER, generator=g))
        scale[h, idx] = s
    return scale


def kv_stream(n_tokens, n_heads, seed, device="cpu"):
    """[n_heads, n_tokens, 128] bf16: N(0,1) with 4 outlier channels per head."""
    scale = outlier_profile(n_heads, seed).to(device)
    x = torch.randn(n_heads, n_tokens, D, generator=_gen(seed + 7919, device), device=device, dtype=torch.float32)
    x.mul_(scale[:, None, :])
    return x.to(torch.bfloat16)


def queries(batch, n_q_heads, seed, device="cpu"):
    """[batch, n_q_heads, 128] bf16, i.i.d. N(0, 1)."""
    x = torch.randn(batch, n_q_heads, D, generator=_gen(seed + 104729, device), device=device, dtype=torch.float32)
    return x.to(torch.bfloat16)


def ragged_lengths(n_seq, lo, hi, seed):
    """n_seq context lengths, uniform integers in [lo, hi] (numpy int32)."""
    rng = np.random.default_rng(int(seed))
    return rng.integers(lo, hi + 1, size=n_seq).astype(np.int32)
