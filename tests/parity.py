"""Helpers for the GPU parity tests: oracle calls on the same rounded inputs, error metrics."""
import numpy as np
import torch


def host(t):
    """Device tensor -> float32 numpy (bf16 / fp32 values are exact in float32)."""
    return t.detach().float().cpu().numpy()


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


def max_rel(got, ref):
    """max |got - ref| / max |ref| (element-wise relative error is undefined at the zeros of a
    signed sum)."""
    got = np.asarray(got, dtype=np.float64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-300))


BF16_REL_L2 = 1e-2      # bf16 inputs, fp32 accumulation
F32_MAX_REL = 1e-4      # fp32 inputs


def oracle_decode(oracle, x, use_r=True, seqs=None):
    """Oracle output [B or len(seqs), Hq, d] for a decode input dict (optionally a subset of
    sequences)."""
    q, r, k, v = x["q"], x["r"], x["k"], x["v"]
    sl = x.get("seq_lens")
    if seqs is not None:
        idx = torch.as_tensor(seqs, device=q.device)
        q, r, k, v = q[idx], r[idx], k[idx], v[idx]
        sl = sl[idx] if sl is not None else None
    qh, rh = host(q)[:, :, None, :], host(r)[:, :, None, :]
    if not use_r:
        rh = np.zeros_like(rh)
    out = oracle.forward(qh, rh, host(k), host(v), x["scale"],
                         seq_lens=None if sl is None else sl.cpu().numpy())
    return out[:, :, 0, :]


def oracle_prefill(oracle, y, causal=True, use_r=True, rows=None):
    q, r, k, v = (host(y[n]) for n in "qrkv")
    if not use_r:
        r = np.zeros_like(r)
    return oracle.forward(q, r, k, v, y["scale"], causal=causal, rows=rows)


def assert_gradient_close(name, got, ref, tol, info=()):
    """rel L2 <= tol over the whole gradient. A reference that is exactly zero (dQ, dR, and with
    them the probe and query terms of dK, of rows that see a single key) has no relative error:
    there the kernel's fp32 rounding residue must stay below 1e-5 rms."""
    got = np.asarray(got, dtype=np.float64)
    assert np.isfinite(got).all(), (name,) + tuple(info)
    ref_norm = np.linalg.norm(ref)
    if ref_norm == 0.0:
        assert np.sqrt(np.mean(got ** 2)) <= 1e-5, (name, "zero reference") + tuple(info)
    else:
        err = np.linalg.norm(got - ref)
        assert err <= tol * ref_norm, (name, err / ref_norm) + tuple(info)
