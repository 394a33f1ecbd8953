"""RMSNorm + rotary position embedding on q, k, rho -- CPU ORACLE in numpy float64 (test
infrastructure, not product).

The paper's language-model runs (experiment setup of Sec. 5 and the backbone appendix) apply
RMSNorm to the q and k vectors of every head, additionally to rho in a Parallax layer, and RoPE
with base theta = 10^6 to q and k (and, where used, to rho with the same base). The paper gives
no formulas; the standard ones of the named architecture are taken:

    RMSNorm over the head dimension:  y = x / sqrt(mean_c(x_c^2) + eps) * gamma
    RoPE at position pos, pairs of adjacent dimensions (2i, 2i + 1) -- the pairing of the
    implementation the paper names (complex pairs) -- with frequency theta^(-2i/d):
        y_2i     = x_2i cos(a) - x_2i+1 sin(a)
        y_2i+1   = x_2i sin(a) + x_2i+1 cos(a),      a = pos * theta^(-2i/d)

Pins (tests/test_oracle_norm_rope.py): a hand-worked two-dimensional rotation, unit RMS,
scale invariance of the norm, position 0 = identity, rotations compose (positions add), and the
property RoPE exists for: (R_m q).(R_n k) depends only on m - n.
"""
from __future__ import annotations

import numpy as np


def rms_norm(x, gamma, eps=1e-6):
    """x [..., d], gamma [d]: x / sqrt(mean(x^2) + eps) * gamma."""
    x = np.asarray(x, dtype=np.float64)
    ms = (x * x).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gamma, dtype=np.float64)


def rope(x, positions, theta=1.0e6):
    """x [..., T, d] with d even, positions [T] (or broadcastable to x.shape[:-1]): rotate the
    adjacent pairs (2i, 2i + 1) by positions * theta^(-2i/d)."""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    assert d % 2 == 0
    freq = theta ** (-np.arange(0, d, 2, dtype=np.float64) / d)              # [d/2]
    ang = np.asarray(positions, dtype=np.float64)[..., None] * freq          # [..., T, d/2]
    c, s = np.cos(ang), np.sin(ang)
    even, odd = x[..., 0::2], x[..., 1::2]
    out = np.empty_like(x)
    out[..., 0::2] = even * c - odd * s
    out[..., 1::2] = even * s + odd * c
    return out


def norm_rope(x, gamma, positions, eps=1e-6, theta=1.0e6):
    """RMSNorm, then RoPE: what the attention kernels expect of q, k and rho."""
    return rope(rms_norm(x, gamma, eps), positions, theta)
