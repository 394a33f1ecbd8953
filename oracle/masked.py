"""Parallax forward under an arbitrary boolean mask -- CPU ORACLE in numpy float64 (test
infrastructure, not product).

The forward equation of the paper (Sec. 3.1, re-weighted softmax form) with the sum over j
restricted to the keys a mask allows -- what "contextual sparsity patterns ... dilated or block
sparse" (Sec. 5) means for this operator: softmax, ubar and the output all run over the allowed
set only. Rows with no allowed key are undefined in the paper and returned as zeros.

    mask [Tq, Lk] (or broadcastable [B, Hq, Tq, Lk]) boolean, True = key allowed

`block_mask_to_dense` expands a block mask over (row block, key tile) to that form, optionally
intersected with the causal set (rows = the last Tq positions).

Pins (tests/test_oracle_masked.py): all-true, causal and banded masks against the C oracle
(which knows those three cases by construction, not through a mask), and for a random mask the
row-by-row equivalence with the C oracle run on the gathered keys.
"""
from __future__ import annotations

import numpy as np


def masked_forward(q, r, k, v, scale, mask):
    q, r, k, v = (np.asarray(x, dtype=np.float64) for x in (q, r, k, v))
    B, Hq, Tq, d = q.shape
    _, Hkv, Lk, _ = k.shape
    G = Hq // Hkv
    mask = np.broadcast_to(np.asarray(mask, dtype=bool), (B, Hq, Tq, Lk))
    out = np.zeros_like(q)
    for b in range(B):
        for h in range(Hq):
            K, V, M = k[b, h // G], v[b, h // G], mask[b, h]
            A = np.where(M, scale * (q[b, h] @ K.T), -np.inf)
            amax = A.max(axis=1, keepdims=True)
            amax = np.where(np.isfinite(amax), amax, 0.0)      # empty rows
            W = np.where(M, np.exp(A - amax), 0.0)
            omega = W.sum(axis=1, keepdims=True)
            P = W / np.where(omega > 0, omega, 1.0)
            U = r[b, h] @ K.T
            ubar = (P * U).sum(axis=1, keepdims=True)
            out[b, h] = (P * (1.0 + ubar - U)) @ V
    return out


def block_mask_to_dense(block_mask, Tq, Lk, block_rows, block_keys, causal):
    """block_mask [..., ceil(Tq / block_rows), ceil(Lk / block_keys)] -> [..., Tq, Lk]."""
    bm = np.asarray(block_mask, dtype=bool)
    dense = np.repeat(np.repeat(bm, block_rows, axis=-2), block_keys, axis=-1)[..., :Tq, :Lk]
    if causal:
        dense = dense & np.tril(np.ones((Tq, Lk), dtype=bool), k=Lk - Tq)
    return dense
