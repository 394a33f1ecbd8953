"""Pins of the backward oracle (oracle/parallax_backward.py, the closed forms of the paper's
App. D) against things that are not itself: finite differences of the C forward oracle,
PyTorch autograd on a float64 transcription of the forward DEFINITION, the textbook softmax
backward at R = 0, conservation laws, and planted mistakes that these pins must reject."""
import numpy as np
import pytest
import torch

from oracle import parallax_backward as pb
from oracle import parallax_oracle as po


def _problem(seed, B=2, Hq=4, Hkv=2, Tq=5, Lk=7, d=3):
    rng = np.random.default_rng(seed)
    q, r = rng.standard_normal((B, Hq, Tq, d)), 0.7 * rng.standard_normal((B, Hq, Tq, d))
    k, v = rng.standard_normal((B, Hkv, Lk, d)), rng.standard_normal((B, Hkv, Lk, d))
    g = rng.standard_normal((B, Hq, Tq, d))
    return q, r, k, v, g


def _finite_differences(q, r, k, v, g, scale, causal, eps=1e-6):
    """d/dx of L = sum(g * forward(x)) by central differences of the C forward oracle."""
    grads = []
    xs = [q, r, k, v]
    for n in range(4):
        x = xs[n]
        out = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = x[idx]
            x[idx] = old + eps
            up = (g * po.forward(*xs, scale, causal=causal)).sum()
            x[idx] = old - eps
            dn = (g * po.forward(*xs, scale, causal=causal)).sum()
            x[idx] = old
            out[idx] = (up - dn) / (2 * eps)
        grads.append(out)
    return grads


@pytest.mark.parametrize("causal,Tq,Lk", [(True, 5, 5), (True, 3, 7), (False, 4, 6)])
def test_closed_forms_match_finite_differences_of_the_forward_oracle(causal, Tq, Lk):
    q, r, k, v, g = _problem(11, B=1, Hq=4, Hkv=2, Tq=Tq, Lk=Lk, d=3)
    want = _finite_differences(q, r, k, v, g, 0.6, causal)
    got = pb.backward(q, r, k, v, g, 0.6, causal=causal)
    for name, a, b in zip(("dq", "dr", "dk", "dv"), got, want):
        np.testing.assert_allclose(a, b, rtol=2e-6, atol=2e-7, err_msg=name)


def _torch_forward(q, r, k, v, scale, causal, window=0):
    """The forward definition (Sec. 3.1, re-weighted softmax form) in PyTorch float64."""
    B, Hq, Tq, d = q.shape
    Hkv, Lk = k.shape[1], k.shape[2]
    G = Hq // Hkv
    kk, vv = k.repeat_interleave(G, dim=1), v.repeat_interleave(G, dim=1)
    a = scale * q @ kk.transpose(-1, -2)
    if causal:
        keep = torch.tril(torch.ones(Tq, Lk, dtype=torch.bool), diagonal=Lk - Tq)
        if window > 0:   # a row sees its own position and the window - 1 before it
            keep &= torch.triu(torch.ones(Tq, Lk, dtype=torch.bool), diagonal=Lk - Tq - (window - 1))
        a = a.masked_fill(~keep, float("-inf"))
    p = torch.softmax(a, dim=-1)
    u = r @ kk.transpose(-1, -2)
    ubar = (p * u).sum(-1, keepdim=True)
    return (p * (1.0 + ubar - u)) @ vv


@pytest.mark.parametrize("causal,Tq,Lk,Hq,Hkv", [(True, 33, 33, 4, 2), (True, 9, 40, 6, 2),
                                                   (False, 17, 29, 4, 4), (True, 1, 12, 8, 1)])
def test_closed_forms_match_autograd_of_the_definition(causal, Tq, Lk, Hq, Hkv):
    q, r, k, v, g = _problem(12, B=2, Hq=Hq, Hkv=Hkv, Tq=Tq, Lk=Lk, d=8)
    tq, tr, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, r, k, v))
    out = _torch_forward(tq, tr, tk, tv, 0.35, causal)
    # the transcription is the same function as the C oracle
    np.testing.assert_allclose(out.detach().numpy(), po.forward(q, r, k, v, 0.35, causal=causal),
                               rtol=1e-11, atol=1e-12)
    (out * torch.tensor(g)).sum().backward()
    got = pb.backward(q, r, k, v, g, 0.35, causal=causal)
    for name, a, t in zip(("dq", "dr", "dk", "dv"), got, (tq, tr, tk, tv)):
        np.testing.assert_allclose(a, t.grad.numpy(), rtol=1e-10, atol=1e-11, err_msg=name)


@pytest.mark.parametrize("Tq,Lk,window", [(12, 12, 1), (12, 12, 4), (9, 20, 5), (7, 7, 50)])
def test_sliding_window_closed_forms_match_autograd_and_finite_differences(Tq, Lk, window):
    """The same closed forms over the window's key set: against autograd of the definition with
    the window written as a band mask, and against central differences of the C forward oracle
    (which has its own window code and its own pins)."""
    q, r, k, v, g = _problem(17, B=1, Hq=4, Hkv=2, Tq=Tq, Lk=Lk, d=3)
    tq, tr, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, r, k, v))
    out = _torch_forward(tq, tr, tk, tv, 0.5, True, window)
    np.testing.assert_allclose(out.detach().numpy(), po.forward(q, r, k, v, 0.5, causal=True, window=window),
                               rtol=1e-11, atol=1e-12)
    (out * torch.tensor(g)).sum().backward()
    got = pb.backward(q, r, k, v, g, 0.5, causal=True, window=window)
    for name, a, t in zip(("dq", "dr", "dk", "dv"), got, (tq, tr, tk, tv)):
        np.testing.assert_allclose(a, t.grad.numpy(), rtol=1e-10, atol=1e-11, err_msg=name)
    if window >= Tq + (Lk - Tq):   # a window that covers everything is no window
        for a, b in zip(got, pb.backward(q, r, k, v, g, 0.5, causal=True)):
            np.testing.assert_array_equal(a, b)
    if window == 1:                # one key per row: o_i = v_i', so dV_i' = sum over heads of dO_i, the rest is zero
        np.testing.assert_allclose(got[0], 0.0, atol=1e-12)
        np.testing.assert_allclose(got[1], 0.0, atol=1e-12)
        np.testing.assert_allclose(got[2], 0.0, atol=1e-12)
        np.testing.assert_allclose(got[3][:, :, Lk - Tq:], g.reshape(1, 2, 2, Tq, 3).sum(axis=2), atol=1e-12)
    o, vbar, ubar, lw = pb.forward_with_cache(q, r, k, v, 0.5, causal=True, window=window)
    np.testing.assert_allclose(o, po.forward(q, r, k, v, 0.5, causal=True, window=window), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(vbar, po.forward(q, np.zeros_like(r), k, v, 0.5, causal=True, window=window),
                               rtol=1e-12, atol=1e-13)


def test_sliding_window_finite_differences():
    q, r, k, v, g = _problem(18, B=1, Hq=2, Hkv=1, Tq=6, Lk=8, d=3)
    xs = [q, r, k, v]
    got = pb.backward(q, r, k, v, g, 0.6, causal=True, window=3)
    eps = 1e-6
    for n in range(4):
        x = xs[n]
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = x[idx]
            x[idx] = old + eps
            up = (g * po.forward(*xs, 0.6, causal=True, window=3)).sum()
            x[idx] = old - eps
            dn = (g * po.forward(*xs, 0.6, causal=True, window=3)).sum()
            x[idx] = old
            assert abs((up - dn) / (2 * eps) - got[n][idx]) <= 2e-6 * max(1.0, abs(got[n][idx])), (n, idx)


def test_zero_probe_is_the_textbook_softmax_backward():
    q, r, k, v, g = _problem(13, B=1, Hq=2, Hkv=2, Tq=6, Lk=6, d=4)
    r = np.zeros_like(r)
    dq, dr, dk, dv = pb.backward(q, r, k, v, g, 0.5, causal=True)
    for h in range(2):
        a = np.where(np.tril(np.ones((6, 6), bool)), 0.5 * q[0, h] @ k[0, h].T, -np.inf)
        p = np.exp(a - a.max(1, keepdims=True))
        p /= p.sum(1, keepdims=True)
        o = p @ v[0, h]
        dp = g[0, h] @ v[0, h].T
        ds = p * (dp - (g[0, h] * o).sum(1, keepdims=True))
        np.testing.assert_allclose(dv[0, h], p.T @ g[0, h], atol=1e-12)
        np.testing.assert_allclose(dq[0, h], 0.5 * ds @ k[0, h], atol=1e-12)
        np.testing.assert_allclose(dk[0, h], 0.5 * ds.T @ q[0, h], atol=1e-12)
        # dR is not zero at R = 0: it is minus the softmax-weighted value/key covariance applied to dO
        kbar, vbar = p @ k[0, h], p @ v[0, h]
        for i in range(6):
            cov = ((v[0, h] - vbar[i]) * p[i][:, None]).T @ (k[0, h] - kbar[i])   # [d_v, d_k]
            np.testing.assert_allclose(dr[0, h, i], -g[0, h, i] @ cov, atol=1e-12)


@pytest.mark.parametrize("causal", [True, False])
def test_conservation_laws(causal):
    """The forward does not change when every key is moved by the same vector, and moves by c
    when every value does: so sum_j dK_j = 0 and sum_j dV_j = sum_i dO_i, per KV head."""
    q, r, k, v, g = _problem(14, B=2, Hq=6, Hkv=2, Tq=9, Lk=9 if causal else 13, d=5)
    dq, dr, dk, dv = pb.backward(q, r, k, v, g, 0.8, causal=causal)
    np.testing.assert_allclose(dk.sum(axis=2), 0.0, atol=1e-11)
    want = g.reshape(2, 2, 3, 9, 5).sum(axis=(2, 3))
    np.testing.assert_allclose(dv.sum(axis=2), want, atol=1e-11)


def test_cache_of_the_forward_matches_the_forward_oracle():
    q, r, k, v, _ = _problem(15, B=2, Hq=4, Hkv=2, Tq=6, Lk=10, d=4)
    o, vbar, ubar, log_omega = pb.forward_with_cache(q, r, k, v, 0.45, causal=True)
    np.testing.assert_allclose(o, po.forward(q, r, k, v, 0.45, causal=True), rtol=1e-12, atol=1e-13)
    # vbar is the forward at R = 0; a one-key row has omega = exp(scale q.k) and ubar = rho.k
    np.testing.assert_allclose(vbar, po.forward(q, np.zeros_like(r), k, v, 0.45, causal=True),
                               rtol=1e-12, atol=1e-13)
    q1, r1 = q[:, :, :1], r[:, :, :1]
    _, _, ub1, lw1 = pb.forward_with_cache(q1, r1, k[:, :, :1], v[:, :, :1], 0.45, causal=True)
    kk = np.repeat(k[:, :, 0], 2, axis=1)
    np.testing.assert_allclose(ub1[:, :, 0], (r1[:, :, 0] * kk).sum(-1), atol=1e-13)
    np.testing.assert_allclose(lw1[:, :, 0], 0.45 * (q1[:, :, 0] * kk).sum(-1), atol=1e-13)


MUTANTS = {
    "g1_without_tau": ("g1 = P * (a - tau + (ubar - U) * delta)", "g1 = P * (a + (ubar - U) * delta)"),
    "g1_probe_term_sign": ("g1 = P * (a - tau + (ubar - U) * delta)", "g1 = P * (a - tau - (ubar - U) * delta)"),
    "g1_uncentred": ("g1 = P * (a - tau + (ubar - U) * delta)", "g1 = P * (a - tau + (ubar - U) * a)"),
    "g2_sign": ("g2 = -P * delta", "g2 = P * delta"),
    "g2_uncentred": ("g2 = -P * delta", "g2 = -P * a"),
    "dq_unscaled": ("dq[b, h] = scale * (g1 @ K)", "dq[b, h] = g1 @ K"),
    "dr_scaled": ("dr[b, h] = g2 @ K", "dr[b, h] = scale * (g2 @ K)"),
    "dk_probe_term_scaled": ("+ g2.T @ r[b, h]", "+ scale * (g2.T @ r[b, h])"),
    "dk_uses_q_twice": ("+ g2.T @ r[b, h]", "+ g2.T @ q[b, h]"),
    "dv_plain_softmax": ("dv[b, hk] += (P * C).T @ d_o[b, h]", "dv[b, hk] += P.T @ d_o[b, h]"),
    "gqa_not_summed": ("dk[b, hk] += scale", "dk[b, hk] = scale"),
    "beta_from_o": ("beta = (d_o[b, h] * vbar)", "beta = (d_o[b, h] * o)"),
}
WINDOW_MUTANTS = {
    "window_one_short": ("mask &= key >= pos - (window - 1)", "mask &= key >= pos - (window - 2)"),
    "window_one_long": ("mask &= key >= pos - (window - 1)", "mask &= key >= pos - window"),
    "window_from_row_index": ("mask &= key >= pos - (window - 1)", "mask &= key >= np.arange(Tq)[:, None] - (window - 1)"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_rejected(name):
    """Each single-token mistake in the closed forms must fail the autograd pin."""
    import inspect

    src = inspect.getsource(pb)
    old, new = MUTANTS[name]
    assert src.count(old) == 1, "mutation site vanished from the oracle source"
    ns = {}
    exec(compile(src.replace(old, new), "<mutant>", "exec"), ns)
    q, r, k, v, g = _problem(16, B=1, Hq=4, Hkv=2, Tq=7, Lk=9, d=4)
    tq, tr, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, r, k, v))
    (_torch_forward(tq, tr, tk, tv, 0.6, True) * torch.tensor(g)).sum().backward()
    got = ns["backward"](q, r, k, v, g, 0.6, causal=True)
    worst = max(np.abs(a - t.grad.numpy()).max() for a, t in zip(got, (tq, tr, tk, tv)))
    assert worst > 1e-6, "no pin noticed the planted mistake '%s'" % name


@pytest.mark.parametrize("name", sorted(WINDOW_MUTANTS))
def test_planted_window_mistake_is_rejected(name):
    import inspect

    src = inspect.getsource(pb)
    old, new = WINDOW_MUTANTS[name]
    assert src.count(old) == 1, "mutation site vanished from the oracle source"
    ns = {}
    exec(compile(src.replace(old, new), "<mutant>", "exec"), ns)
    q, r, k, v, g = _problem(19, B=1, Hq=4, Hkv=2, Tq=7, Lk=11, d=4)
    tq, tr, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, r, k, v))
    (_torch_forward(tq, tr, tk, tv, 0.6, True, 4) * torch.tensor(g)).sum().backward()
    got = ns["backward"](q, r, k, v, g, 0.6, causal=True, window=4)
    worst = max(np.abs(a - t.grad.numpy()).max() for a, t in zip(got, (tq, tr, tk, tv)))
    assert worst > 1e-6, "no pin noticed the planted mistake '%s'" % name
