"""Parallax attention backward -- CPU ORACLE in numpy float64 (test infrastructure, not product).

The closed-form gradients of the paper's App. D ("Parallax Backward"), written out per head with
explicit T x L matrices, in the paper's notation:

    w_ij = exp(q_i.k_j / h)  (scale = 1/h),  omega_i = sum_j w_ij,  p_ij = w_ij / omega_i
    u_ij = rho_i.k_j         (t_ij of the paper up to the j-independent rho_i.q_i, which cancels
                              in tbar_i - t_ij = ubar_i - u_ij)
    o_i    = sum_j p_ij (1 + ubar_i - u_ij) v_j          (re-weighted softmax form)
    vbar_i = sum_j p_ij v_j
    tau_i  = dO_i.o_i,  beta_i = dO_i.vbar_i,  a_ij = dO_i.v_j,  delta_ij = a_ij - beta_i
    g1_ij  = p_ij [a_ij - tau_i + (ubar_i - u_ij) delta_ij],     g2_ij = -p_ij delta_ij
    dQ_i = scale * sum_j g1_ij k_j          dR_i = sum_j g2_ij k_j
    dK_j = scale * sum_i g1_ij q_i + sum_i g2_ij rho_i
    dV_j = sum_i p_ij (1 + ubar_i - u_ij) dO_i

The sums run over the allowed (row, key) pairs: causal with the rows as the last Tq positions
(key j allowed iff j <= i + (Lk - Tq)), else every key; with a sliding window of W > 0 (causal
only) a row also does not see keys before its own position minus W - 1. GQA: the gradients of a KV head add up
over the query heads of its group. No tiling, no recomputation tricks: every matrix is formed.

Pins (tests/test_oracle_backward.py): central finite differences of the forward oracle (the C
file, which shares nothing with this one), automatic differentiation of a plain PyTorch float64
transcription of the forward definition, the textbook softmax-attention backward at R = 0, and
the two conservation laws that follow from the forward's invariances (key translation:
sum_j dK_j = 0; value translation: sum_j dV_j = sum_i dO_i per KV head).
"""
from __future__ import annotations

import numpy as np


def _mask(Tq, Lk, causal, window=0):
    if not causal:
        assert window == 0, "a sliding window is defined for causal attention"
        return np.ones((Tq, Lk), dtype=bool)
    pos = np.arange(Tq)[:, None] + (Lk - Tq)               # the row's own position among the keys
    key = np.arange(Lk)[None, :]
    mask = key <= pos
    if window > 0:
        mask &= key >= pos - (window - 1)                  # itself and the window - 1 positions before it
    return mask


def forward_with_cache(q, r, k, v, scale, causal=True, window=0):
    """Forward by the definition plus the per-row cache the paper's backward reads:
    o, vbar [B, Hq, Tq, d]; ubar, log_omega (natural log of sum_j exp(scale q.k)) [B, Hq, Tq]."""
    q, r, k, v = (np.asarray(x, dtype=np.float64) for x in (q, r, k, v))
    B, Hq, Tq, d = q.shape
    _, Hkv, Lk, _ = k.shape
    G = Hq // Hkv
    mask = _mask(Tq, Lk, causal, window)
    o, vbar = np.zeros_like(q), np.zeros_like(q)
    ubar, log_omega = np.zeros((B, Hq, Tq)), np.zeros((B, Hq, Tq))
    for b in range(B):
        for h in range(Hq):
            K, V = k[b, h // G], v[b, h // G]
            A = np.where(mask, scale * (q[b, h] @ K.T), -np.inf)
            amax = A.max(axis=1, keepdims=True)
            W = np.exp(A - amax)
            omega = W.sum(axis=1, keepdims=True)
            P = W / omega
            U = r[b, h] @ K.T
            ub = (P * U).sum(axis=1, keepdims=True)
            o[b, h] = (P * (1.0 + ub - U)) @ V
            vbar[b, h] = P @ V
            ubar[b, h] = ub[:, 0]
            log_omega[b, h] = (amax + np.log(omega))[:, 0]
    return o, vbar, ubar, log_omega


def backward(q, r, k, v, d_o, scale, causal=True, window=0):
    """dQ, dR [B, Hq, Tq, d] and dK, dV [B, Hkv, Lk, d] by the closed forms of App. D."""
    q, r, k, v, d_o = (np.asarray(x, dtype=np.float64) for x in (q, r, k, v, d_o))
    B, Hq, Tq, d = q.shape
    _, Hkv, Lk, _ = k.shape
    G = Hq // Hkv
    mask = _mask(Tq, Lk, causal, window)
    dq, dr = np.zeros_like(q), np.zeros_like(q)
    dk, dv = np.zeros_like(k), np.zeros_like(k)
    for b in range(B):
        for h in range(Hq):
            hk = h // G
            K, V = k[b, hk], v[b, hk]
            A = np.where(mask, scale * (q[b, h] @ K.T), -np.inf)
            W = np.exp(A - A.max(axis=1, keepdims=True))
            P = W / W.sum(axis=1, keepdims=True)           # p_ij, zero outside the mask
            U = r[b, h] @ K.T                              # u_ij
            ubar = (P * U).sum(axis=1, keepdims=True)
            C = 1.0 + ubar - U                             # 1 + tbar_i - t_ij
            o = (P * C) @ V
            vbar = P @ V
            tau = (d_o[b, h] * o).sum(axis=1, keepdims=True)
            beta = (d_o[b, h] * vbar).sum(axis=1, keepdims=True)
            a = d_o[b, h] @ V.T                            # a_ij
            delta = a - beta
            g1 = P * (a - tau + (ubar - U) * delta)
            g2 = -P * delta
            dq[b, h] = scale * (g1 @ K)
            dr[b, h] = g2 @ K
            dk[b, hk] += scale * (g1.T @ q[b, h]) + g2.T @ r[b, h]
            dv[b, hk] += (P * C).T @ d_o[b, h]
    return dq, dr, dk, dv
