"""Parallax decode over an MLA-style latent cache -- CPU ORACLE in numpy float64 (test
infrastructure, not product).

The paper only states that Parallax is structurally compatible with multi-head latent attention
(closing discussion, "Optimizing the efficiency of Parallax"). The reading taken here is the
usual absorbed-projection decode form of such a cache: every token stores ONE row
c_j = [latent (d_c) | rope part (d_r)] shared by all heads; with the up-projections absorbed
into the queries, head h scores a token with the whole row and reads its value from the latent
part only:

    key_j   = c_j            (d_c + d_r numbers)
    value_j = c_j[:d_c]
    a_hj = scale * q_h . c_j,  p_hj = softmax_j(a_hj),  u_hj = rho_h . c_j,  ubar_h = sum_j p_hj u_hj
    o_h  = sum_j p_hj (1 + ubar_h - u_hj) c_j[:d_c]       (the forward definition of Sec. 3.1)

q, rho are [B, Hq, d_c + d_r] (already in the latent space), the output is [B, Hq, d_c] (the
value up-projection is applied outside). Written with explicit per-head vectors, no tiling.

`mla_rows` is the same for Tq query rows per head that sit at the LAST Tq positions of the
cached sequence (several rows of a speculative / chunked decode step, or -- with Tq = the prompt
length -- the causal prefill over the latent cache): row t sees the tokens 0 .. n - Tq + t, and
with a sliding window of W > 0 only the last W of those (its own position and the W - 1 before).
A row that sees no token returns zeros.

Pins (tests/test_oracle_mla.py): equality with the C forward oracle run on one shared KV head
whose values are the latent part padded with zeros (a different program, with its own pins);
rho = 0 against a library softmax attention whose value width differs from its key width; a
two-token closed form; invariance under a common shift of the rope part of every key.
"""
from __future__ import annotations

import numpy as np


def mla_decode(q, r, ckv, d_latent, scale, seq_lens=None):
    """q, r [B, Hq, dk]; ckv [B, L, dk]; returns o [B, Hq, d_latent]. Sequence b uses its first
    seq_lens[b] rows (all L without seq_lens); an empty sequence returns zeros."""
    q, r, ckv = (np.asarray(x, dtype=np.float64) for x in (q, r, ckv))
    B, Hq, dk = q.shape
    L = ckv.shape[1]
    assert ckv.shape == (B, L, dk) and r.shape == q.shape and 0 < d_latent <= dk
    out = np.zeros((B, Hq, d_latent))
    for b in range(B):
        n = L if seq_lens is None else int(seq_lens[b])
        if n <= 0:
            continue
        keys = ckv[b, :n]                    # [n, dk]
        values = ckv[b, :n, :d_latent]       # [n, d_latent]
        for h in range(Hq):
            a = scale * (keys @ q[b, h])
            w = np.exp(a - a.max())
            p = w / w.sum()
            u = keys @ r[b, h]
            ubar = p @ u
            out[b, h] = (p * (1.0 + ubar - u)) @ values
    return out


def mla_rows(q, r, ckv, d_latent, scale, seq_lens=None, window=0):
    """q, r [B, Hq, Tq, dk]; ckv [B, L, dk]; returns o [B, Hq, Tq, d_latent]. Row t of sequence b
    (n = seq_lens[b] tokens) is at position n - Tq + t and sees the tokens j with
    max(0, pos - window + 1) <= j <= pos (window = 0: from token 0)."""
    q, r, ckv = (np.asarray(x, dtype=np.float64) for x in (q, r, ckv))
    B, Hq, Tq, dk = q.shape
    L = ckv.shape[1]
    assert ckv.shape == (B, L, dk) and r.shape == q.shape and 0 < d_latent <= dk and window >= 0
    out = np.zeros((B, Hq, Tq, d_latent))
    for b in range(B):
        n = L if seq_lens is None else int(seq_lens[b])
        for t in range(Tq):
            pos = n - Tq + t
            first = max(0, pos - window + 1) if window > 0 else 0
            if pos < first:
                continue                          # (pos < 0: the row lies before the sequence)
            keys = ckv[b, first:pos + 1]
            values = keys[:, :d_latent]
            for h in range(Hq):
                a = scale * (keys @ q[b, h, t])
                w = np.exp(a - a.max())
                p = w / w.sum()
                u = keys @ r[b, h, t]
                ubar = p @ u
                out[b, h, t] = (p * (1.0 + ubar - u)) @ values
    return out
