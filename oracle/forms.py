"""Second and third forms of the Parallax forward in numpy float64 (test infrastructure).

* ``covariance_form``  -- o = vbar - Sigma_KV rho, the right-hand side of the paper's
  forward equation (Sec. 3.1), with the d x d softmax-weighted KV covariance formed
  explicitly.
* ``streaming_*``      -- the forward as a fold over keys. From the re-weighted softmax form
  of Sec. 3.1, o = sum_j p_j (1 + ubar - u_j) v_j with p_j = w_j / omega, everything a row
  needs from a set J of keys is five moments of the unnormalised weights w_j = 2^(a_j - lam)
  (a_j = scale * log2(e) * q.k_j, lam any reference):
      omega = sum w_j,  mu = sum w_j u_j,  Mv = sum w_j v_j,  Muv = sum w_j u_j v_j
  and then  o = Mv / omega * (1 + mu / omega) - Muv / omega.  The state (lam, omega, mu, Mv, Muv)
  of one key is (a_j, 1, u_j, v_j, u_j v_j); the states of disjoint key sets merge by bringing
  both to the larger reference and adding (``merge_states``). A split-KV workspace record
  (Sec. 3.3, App. C) is exactly such a state for the keys of the split, which is what the tests
  compare the kernels' records with; tiling enters only through the order of the merges.

The user-facing ``scale`` is 1/h of the natural exponential exp(q.k/h); states are kept in the
base-2 domain (a_j carries the factor log2 e), as the split records are.

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


def _key_state(Qr, Rr, kj, vj, s, allowed):
    """State of the single key j for every row: (a_j, 1, u_j, v_j, u_j v_j), or the empty state
    (-inf, 0, 0, 0, 0) for rows that may not see the key."""
    lam = np.where(allowed, s * (Qr @ kj), -np.inf)
    w = allowed.astype(np.float64)
    u = w * (Rr @ kj)
    return lam, w, u, w[:, None] * vj[None, :], u[:, None] * vj[None, :]


def merge_states(A, B):
    """States of two disjoint key sets -> state of their union: both are brought to the larger
    reference, then the moments add. The empty state is the neutral element."""
    lam = np.maximum(A[0], B[0])
    safe = np.where(np.isfinite(lam), lam, 0.0)
    fa = np.where(np.isfinite(A[0]), np.exp2(A[0] - safe), 0.0)
    fb = np.where(np.isfinite(B[0]), np.exp2(B[0] - safe), 0.0)
    return (lam, fa * A[1] + fb * B[1], fa * A[2] + fb * B[2],
            fa[:, None] * A[3] + fb[:, None] * B[3], fa[:, None] * A[4] + fb[:, None] * B[4])


def _empty_state(rows, dv):
    return np.full(rows, -np.inf), np.zeros(rows), np.zeros(rows), np.zeros((rows, dv)), np.zeros((rows, dv))


def streaming_partial(Qr, Rr, K, V, scale, tile, key_lo, key_hi, row_limit=None):
    """State (lam, omega, mu, Mv, Muv) of the keys [key_lo, key_hi) for every row, built key by
    key: the keys of a group of ``tile`` are merged among themselves first, the group then joins
    the running state (any grouping gives the same state up to rounding -- the tests vary it).

    Qr, Rr : [rows, d]; K, V : [L, d]. row_limit[row] (optional) = number of allowed keys
    for that row: it sees the keys j < row_limit[row] (causal / ragged masking).
    """
    rows = Qr.shape[0]
    s = scale * LOG2E
    limit = None if row_limit is None else np.asarray(row_limit)
    total = _empty_state(rows, V.shape[1])
    for c0 in range(key_lo, key_hi, tile):
        group = _empty_state(rows, V.shape[1])
        for j in range(c0, min(c0 + tile, key_hi)):
            allowed = np.ones(rows, dtype=bool) if limit is None else (j < limit)
            group = merge_states(group, _key_state(Qr, Rr, K[j], V[j], s, allowed))
        total = merge_states(total, group)
    return total


def merge_partials(parts):
    """States of the splits of one row block -> state of all keys (the merge of App. C)."""
    total = parts[0]
    for part in parts[1:]:
        total = merge_states(total, part)
    return total


def finalize(state):
    """o = Mv / omega * (1 + mu / omega) - Muv / omega (the re-weighted softmax form of Sec. 3.1
    written in the five moments)."""
    _, omega, mu, Mv, Muv = state
    return (Mv / omega[:, None]) * (1.0 + mu / omega)[:, None] - Muv / omega[:, None]


def streaming_form(q, r, k, v, scale, causal=False, seq_lens=None, tile=16, row_block=8,
                   split_points=None):
    """Whole forward as a fold over keys with split merge. ``split_points`` is an increasing
    list of key indices cutting [0, Lk) into parts (empty parts allowed)."""
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
