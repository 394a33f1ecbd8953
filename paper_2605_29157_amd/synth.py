"""Seeded synthetic inputs for the Parallax attention benchmarks and tests.

This module only draws random tensors in the shapes and distributions of the benchmark
configurations (i.i.d. N(0,1) Q/R/K/V, optional per-(batch, kv-head) key mean offset,
optional probe scaling, ragged lengths uniform in [L/2, L]). It contains none of the
attention arithmetic, so both the CPU oracle's tests and the HIP path may use it.
"""
from __future__ import annotations

import math

import torch


def _randn(shape, gen, device, dtype):
    # draw in fp32 on the generator's device, then round once to the storage dtype
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32).to(dtype)


def _generator(seed: int, device):
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    return gen


def ragged_lengths(B: int, L: int, seed: int) -> torch.Tensor:
    """One integer length per sequence, uniform on [L/2, L] inclusive (CPU int32)."""
    gen = _generator(seed + 7919, "cpu")
    lo = max(1, L // 2)
    return torch.randint(lo, L + 1, (B,), generator=gen, dtype=torch.int64).to(torch.int32)


def decode_inputs(B, Hq, Hkv, L, d, seed, dtype=torch.bfloat16, device="cpu", ragged=False,
                  r_scale=1.0):
    """q, r: [B, Hq, d]; k, v: [B, Hkv, L, d]; seq_lens: int32 [B] or None; scale = 1/sqrt(d)."""
    gen = _generator(seed, device)
    q = _randn((B, Hq, d), gen, device, dtype)
    r = (_randn((B, Hq, d), gen, device, torch.float32) * r_scale).to(dtype)
    k = torch.empty((B, Hkv, L, d), device=device, dtype=dtype)
    v = torch.empty((B, Hkv, L, d), device=device, dtype=dtype)
    for b in range(B):  # per-sequence draws keep the fp32 staging buffer small
        k[b] = _randn((Hkv, L, d), gen, device, dtype)
        v[b] = _randn((Hkv, L, d), gen, device, dtype)
    seq_lens = ragged_lengths(B, L, seed).to(device) if ragged else None
    return dict(q=q, r=r, k=k, v=v, seq_lens=seq_lens, scale=1.0 / math.sqrt(d))


def prefill_inputs(B, Hq, Hkv, T, d, seed, dtype=torch.bfloat16, device="cpu",
                   k_offset_sigma=0.0, r_scale=1.0):
    """q, r: [B, Hq, T, d]; k, v: [B, Hkv, T, d]; scale = 1/sqrt(d).

    k_offset_sigma > 0 adds one offset vector c ~ N(0, sigma^2 I_d) per (batch, kv head) to
    every key row of that head, so the key-centring part of the correction is exercised.
    """
    gen = _generator(seed, device)
    q = _randn((B, Hq, T, d), gen, device, dtype)
    r = (_randn((B, Hq, T, d), gen, device, torch.float32) * r_scale).to(dtype)
    kf = torch.randn((B, Hkv, T, d), generator=gen, device=device, dtype=torch.float32)
    if k_offset_sigma > 0.0:
        off = torch.randn((B, Hkv, 1, d), generator=gen, device=device, dtype=torch.float32)
        kf = kf + k_offset_sigma * off
    k = kf.to(dtype)
    del kf
    v = _randn((B, Hkv, T, d), gen, device, dtype)
    return dict(q=q, r=r, k=k, v=v, scale=1.0 / math.sqrt(d))
