"""Parallax forward under an arbitrary boolean mask -- CPU ORACLE in numpy float64 (test
infrastructure, not product).

The forward equation of the paper (Sec. 3.1, re-weighted softmax form) with the sum over j
restricted to the keys a mask allows -- what "contextual sparsity patterns ... dilated or block
sparse" (Sec. 5) means for this operator: softmax, ubar and the output all run over the allowed
set only. Rows with no allowed key are undefined in the paper and returned as zeros.

    mask [Tq, Lk] (or broadcastable [B, Hq, Tq, Lk]) boolean, True = key allowed

`block_mask_to_dense` expands a block mask over (row block, key tile) to that form, optionally
intersected with the causal set (rows = the last Tq positions).

`masked_backward` is the backward of App. D ("Parallax Backward") with every sum over j (in the
row quantities ubar, vbar, o, dQ, dR) and over i (in dK, dV) restricted to the allowed pairs --
the closed forms do not care which pairs are allowed, only that p_ij = 0 outside. Rows with no
allowed key take no part: their gradients are zero.

Pins (tests/test_oracle_masked.py): all-true, causal and banded masks against the C oracle
(which knows those three cases by construction, not through a mask), and for a random mask the
row-by-row equivalence with the C oracle run on the gathered keys. Backward: automatic
differentiation of a plain PyTorch float64 transcription of the masked definition, central
finite differences of `masked_forward`, the dense / causal / banded cases against
oracle/parallax_backward.py, and the two conservation laws (sum_j dK_j = 0,
sum_j dV_j = sum of dO over the rows that see a key).
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


def masked_forward_with_cache(q, r, k, v, scale, mask):
    """o, vbar [B, Hq, Tq, d] and ubar, log_omega [B, Hq, Tq] (natural log of the masked sum of
    exp(scale q.k); -inf for a row with no allowed key, whose other entries are zero)."""
    q, r, k, v = (np.asarray(x, dtype=np.float64) for x in (q, r, k, v))
    B, Hq, Tq, d = q.shape
    _, Hkv, Lk, _ = k.shape
    G = Hq // Hkv
    mask = np.broadcast_to(np.asarray(mask, dtype=bool), (B, Hq, Tq, Lk))
    o, vbar = np.zeros_like(q), np.zeros_like(q)
    ubar, log_omega = np.zeros((B, Hq, Tq)), np.zeros((B, Hq, Tq))
    for b in range(B):
        for h in range(Hq):
            K, V, M = k[b, h // G], v[b, h // G], mask[b, h]
            A = np.where(M, scale * (q[b, h] @ K.T), -np.inf)
            amax = A.max(axis=1, keepdims=True)
            amax = np.where(np.isfinite(amax), amax, 0.0)
            W = np.where(M, np.exp(A - amax), 0.0)
            omega = W.sum(axis=1, keepdims=True)
            P = W / np.where(omega > 0, omega, 1.0)
            U = r[b, h] @ K.T
            ub = (P * U).sum(axis=1, keepdims=True)
            o[b, h] = (P * (1.0 + ub - U)) @ V
            vbar[b, h] = P @ V
            ubar[b, h] = ub[:, 0]
            with np.errstate(divide="ignore"):
                log_omega[b, h] = (amax + np.log(omega))[:, 0]
    return o, vbar, ubar, log_omega


def masked_backward(q, r, k, v, d_o, scale, mask):
    """dQ, dR [B, Hq, Tq, d] and dK, dV [B, Hkv, Lk, d]: the closed forms of App. D,
        tau_i = dO_i.o_i, beta_i = dO_i.vbar_i, a_ij = dO_i.v_j, delta_ij = a_ij - beta_i
        g1_ij = p_ij [a_ij - tau_i + (ubar_i - u_ij) delta_ij],  g2_ij = -p_ij delta_ij
        dQ_i = scale sum_j g1_ij k_j,  dR_i = sum_j g2_ij k_j
        dK_j = scale sum_i g1_ij q_i + sum_i g2_ij rho_i,  dV_j = sum_i p_ij (1 + ubar_i - u_ij) dO_i
    with p_ij = 0 outside the mask. GQA: a KV head collects from the query heads of its group."""
    q, r, k, v, d_o = (np.asarray(x, dtype=np.float64) for x in (q, r, k, v, d_o))
    B, Hq, Tq, d = q.shape
    _, Hkv, Lk, _ = k.shape
    G = Hq // Hkv
    mask = np.broadcast_to(np.asarray(mask, dtype=bool), (B, Hq, Tq, Lk))
    dq, dr = np.zeros_like(q), np.zeros_like(q)
    dk, dv = np.zeros_like(k), np.zeros_like(k)
    for b in range(B):
        for h in range(Hq):
            hk = h // G
            K, V, M = k[b, hk], v[b, hk], mask[b, h]
            A = np.where(M, scale * (q[b, h] @ K.T), -np.inf)
            amax = A.max(axis=1, keepdims=True)
            amax = np.where(np.isfinite(amax), amax, 0.0)
            W = np.where(M, np.exp(A - amax), 0.0)
            omega = W.sum(axis=1, keepdims=True)
            P = W / np.where(omega > 0, omega, 1.0)        # zero rows where no key is allowed
            U = r[b, h] @ K.T
            ubar = (P * U).sum(axis=1, keepdims=True)
            C = 1.0 + ubar - U
            o = (P * C) @ V
            vbar = P @ V
            tau = (d_o[b, h] * o).sum(axis=1, keepdims=True)
            beta = (d_o[b, h] * vbar).sum(axis=1, keepdims=True)
            a = d_o[b, h] @ V.T
            delta = a - beta
            g1 = P * (a - tau + (ubar - U) * delta)
            g2 = -P * delta
            dq[b, h] = scale * (g1 @ K)
            dr[b, h] = g2 @ K
            dk[b, hk] += scale * (g1.T @ q[b, h]) + g2.T @ r[b, h]
            dv[b, hk] += (P * C).T @ d_o[b, h]
    return dq, dr, dk, dv


def block_mask_to_dense(block_mask, Tq, Lk, block_rows, block_keys, causal):
    """block_mask [..., ceil(Tq / block_rows), ceil(Lk / block_keys)] -> [..., Tq, Lk]."""
    bm = np.asarray(block_mask, dtype=bool)
    dense = np.repeat(np.repeat(bm, block_rows, axis=-2), block_keys, axis=-1)[..., :Tq, :Lk]
    if causal:
        dense = dense & np.tril(np.ones((Tq, Lk), dtype=bool), k=Lk - Tq)
    return dense
