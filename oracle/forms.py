"""Second and third forms of the Parallax forward in numpy float64 (test infrastructure).

* ``covariance_form``  -- o = vbar - Sigma_KV rho, the right-hand side of the paper's
  forward equation (Sec. 3.1), with the d x d softmax-weighted KV covariance formed
  explicitly.
* ``streaming_*``      -- the tile loop of Algorithm 1 (Sec. 3.3) taken step by step in the
  paper's notation (S1, m, alpha, P1, S2, P2, d1, d2, O1, O2), with tile size and split
  boundaries as parameters, plus the split merge and final formula of App. C
  ("in-kernel reduction": log-sum-exp rescale of the partials (m, d1, d2, O1, O2), then
  O1/d1 * (1 + d2/d1) - O2/d1).

Reading taken where the listing is ambiguous: the listing exponentiates with exp2 while
the definition uses exp(q.k/h); the user-facing ``scale`` is 1/h for the natural
exponential and the loop multiplies it by log2(e) before using exp2.

These are used by the tests to check that the three forms agree for any tiling / split
(an algebraic identity of the paper) and as the reference for what a split-KV workspace
must contain. The primary oracle is the C file; nothing here is used by the product.
"""
from __future__ import annotations

import numpy as np

LOG2E = 1.4426950408889634


def _allowed(i, Lk, causal, len_b, Tq=None):
    """Number of allowed keys of query row i; causal rows are the last Tq positions of Lk."""
    if causal:
        return i + 1 + (Lk - (Lk if Tq is None else Tq))
    return min(len_b, Lk)


def covariance_form(q, r, k, v, scale, causal=False, seq_lens=None):
    """o_i = vbar_i - Sigma_KV^(i) rho_i with Sigma_KV = E_p[(v - vbar)(k - kbar)^T]."""
    q, r, k, v = (np.asarray(x, dtype=np.float64) for x in (q, r, k, v))
    B, Hq, Tq, d = q.shape
    _, Hkv, Lk, _ = k.shape
    G = Hq // Hkv
    out = np.zeros_like(q)
    for b in range(B):
        for h in range(Hq):
            kb, vb = k[b, h // G], v[b, h // G]
            for i in range(Tq):
                n = _allowed(i, Lk, causal, Lk if seq_lens is None else int(seq_lens[b]), Tq)
                if n <= 0:
                    continue
                kk, vv = kb[:n], vb[:n]
                a = scale * (kk @ q[b, h, i])
                w = np.exp(a - a.max())
                p = w / w.sum()
                kbar = p @ kk
                vbar = p @ vv
                sigma_kv = (vv - vbar).T @ (p[:, None] * (kk - kbar))  # [d_v, d_k]
                out[b, h, i] = vbar - sigma_kv @ r[b, h, i]
    return out


def streaming_partial(Qr, Rr, K, V, scale, tile, key_lo, key_hi, row_limit=None):
    """Algorithm 1's loop over the keys [key_lo, key_hi) in column tiles of ``tile``.

    Qr, Rr : [rows, d]; K, V : [L, d]. row_limit[row] (optional) = number of allowed keys
    for that row (causal / ragged masking is applied to S1 as the listing's comment says).
    Returns the unnormalised running state (m, d1, d2, O1, O2) in the exp2 domain.
    """
    rows, d = Qr.shape
    s = scale * LOG2E
    m_r = np.full(rows, -np.inf)
    d1 = np.zeros(rows)
    d2 = np.zeros(rows)
    O1 = np.zeros((rows, V.shape[1]))
    O2 = np.zeros((rows, V.shape[1]))
    c0 = key_lo
    while c0 < key_hi:
        c1 = min(c0 + tile, key_hi)
        Kc, Vc = K[c0:c1], V[c0:c1]
        S1 = (Qr @ Kc.T) * s
        if row_limit is not None:
            cols = np.arange(c0, c1)[None, :]
            S1 = np.where(cols < np.asarray(row_limit)[:, None], S1, -np.inf)
        m = np.maximum(m_r, S1.max(axis=1))
        # rows that have seen no allowed key yet keep m = -inf; alpha and P1 are 0 there
        safe_m = np.where(np.isfinite(m), m, 0.0)
        alpha = np.where(np.isfinite(m_r), np.exp2(m_r - safe_m), 0.0)
        P1 = np.exp2(S1 - safe_m[:, None])
        P1 = np.where(np.isfinite(S1), P1, 0.0)
        m_r = m
        S2 = Rr @ Kc.T
        P2 = np.where(P1 > 0.0, P1 * S2, 0.0)
        d1 = alpha * d1 + P1.sum(axis=1)
        d2 = alpha * d2 + P2.sum(axis=1)
        O1 = alpha[:, None] * O1 + P1 @ Vc
        O2 = alpha[:, None] * O2 + P2 @ Vc
        c0 = c1
    return m_r, d1, d2, O1, O2


def merge_partials(parts):
    """Log-sum-exp merge of split partials (App. C, in-kernel reduction)."""
    ms = np.stack([p[0] for p in parts])  # [S, rows]
    m_star = ms.max(axis=0)
    safe = np.where(np.isfinite(m_star), m_star, 0.0)
    d1 = d2 = O1 = O2 = 0.0
    for (m, a1, a2, A1, A2) in parts:
        w = np.where(np.isfinite(m), np.exp2(m - safe), 0.0)
        d1 = d1 + w * a1
        d2 = d2 + w * a2
        O1 = O1 + w[:, None] * A1
        O2 = O2 + w[:, None] * A2
    return m_star, d1, d2, O1, O2


def finalize(state):
    """Last line of Algorithm 1: O = O1/d1 * (1 + d2/d1) - O2/d1."""
    _, d1, d2, O1, O2 = state
    return (O1 / d1[:, None]) * (1.0 + d2 / d1)[:, None] - O2 / d1[:, None]


def streaming_form(q, r, k, v, scale, causal=False, seq_lens=None, tile=16, row_block=8,
                   split_points=None):
    """Whole forward through Algorithm 1 + split merge. ``split_points`` is an increasing list
    of key indices cutting [0, Lk) into parts (empty parts allowed)."""
    q, r, k, v = (np.asarray(x, dtype=np.float64) for x in (q, r, k, v))
    B, Hq, Tq, d = q.shape
    _, Hkv, Lk, _ = k.shape
    G = Hq // Hkv
    cuts = [0] + list(split_points or []) + [Lk]
    out = np.zeros_like(q)
    for b in range(B):
        len_b = Lk if seq_lens is None else int(seq_lens[b])
        for h in range(Hq):
            kb, vb = k[b, h // G], v[b, h // G]
            for r0 in range(0, Tq, row_block):
                r1 = min(r0 + row_block, Tq)
                limit = [(_allowed(i, Lk, causal, len_b, Tq)) for i in range(r0, r1)]
                parts = [
                    streaming_partial(q[b, h, r0:r1], r[b, h, r0:r1], kb, vb, scale, tile,
                                      cuts[s], cuts[s + 1], row_limit=limit)
                    for s in range(len(cuts) - 1)
                ]
                out[b, h, r0:r1] = finalize(merge_partials(parts))
    return out
