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


def paged_cache(x, page_size, seed, spare_pages=3):
    """Scatter the contiguous caches x["k"], x["v"] [B, Hkv, L, d] into page pools
    [num_pages, Hkv, page_size, d] in a seeded random page order (plus a few unused pages) and
    return (k_pool, v_pool, block_table [B, pages per sequence] int32). Layout only."""
    k, v = x["k"], x["v"]
    B, Hkv, L, d = k.shape
    per_seq = (L + page_size - 1) // page_size
    n_pages = B * per_seq + spare_pages
    g = torch.Generator(device="cpu").manual_seed(seed)
    order = torch.randperm(n_pages, generator=g)[: B * per_seq].reshape(B, per_seq)
    pad = per_seq * page_size - L
    kp = torch.nn.functional.pad(k, (0, 0, 0, pad)).reshape(B, Hkv, per_seq, page_size, d)
    vp = torch.nn.functional.pad(v, (0, 0, 0, pad)).reshape(B, Hkv, per_seq, page_size, d)
    k_pool = torch.zeros(n_pages, Hkv, page_size, d, dtype=k.dtype, device=k.device)
    v_pool = torch.zeros_like(k_pool)
    idx = order.reshape(-1).to(k.device)
    k_pool[idx] = kp.permute(0, 2, 1, 3, 4).reshape(B * per_seq, Hkv, page_size, d)
    v_pool[idx] = vp.permute(0, 2, 1, 3, 4).reshape(B * per_seq, Hkv, page_size, d)
    return k_pool, v_pool, order.to(torch.int32).to(k.device)


def mla_decode_inputs(B, Hq, L, seed, d_latent=512, d_rope=64, dtype=torch.bfloat16, device="cpu",
                      ragged=False, r_scale=1.0):
    """q, r: [B, Hq, d_latent + d_rope]; ckv: [B, L, d_latent + d_rope] (one latent | rope row per
    token, shared by all heads); seq_lens: int32 [B] or None; scale = 1/sqrt(d_latent + d_rope)."""
    gen = _generator(seed, device)
    dk = d_latent + d_rope
    q = _randn((B, Hq, dk), gen, device, dtype)
    r = (_randn((B, Hq, dk), gen, device, torch.float32) * r_scale).to(dtype)
    ckv = torch.empty((B, L, dk), device=device, dtype=dtype)
    for b in range(B):  # per sequence: bounds the fp32 temporary
        ckv[b] = _randn((L, dk), gen, device, dtype)
    out = {"q": q, "r": r, "ckv": ckv, "scale": 1.0 / math.sqrt(dk), "d_latent": d_latent}
    if ragged:
        out["seq_lens"] = ragged_lengths(B, L, seed).to(device)
    return out


def mla_paged_cache(x, page_size, seed, spare_pages=3):
    """Scatter the contiguous latent cache x["ckv"] [B, L, dk] into a page pool
    [num_pages, page_size, dk] in a seeded random page order (plus a few unused pages) and return
    (pool, block_table [B, pages per sequence] int32). Layout only."""
    c = x["ckv"]
    B, L, dk = c.shape
    per_seq = (L + page_size - 1) // page_size
    n_pages = B * per_seq + spare_pages
    g = torch.Generator(device="cpu").manual_seed(seed)
    order = torch.randperm(n_pages, generator=g)[: B * per_seq].reshape(B, per_seq)
    pad = per_seq * page_size - L
    cp = torch.nn.functional.pad(c, (0, 0, 0, pad)).reshape(B * per_seq, page_size, dk)
    pool = torch.zeros(n_pages, page_size, dk, dtype=c.dtype, device=c.device)
    pool[order.reshape(-1).to(c.device)] = cp
    return pool, order.to(torch.int32).to(c.device)
