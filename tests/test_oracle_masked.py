"""Pins of the arbitrary-mask oracle (oracle/masked.py) against the C oracle."""
import numpy as np

from oracle import masked
from oracle import parallax_oracle as po


def _problem(seed, B=2, Hq=4, Hkv=2, Tq=9, Lk=14, d=5):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((B, Hq, Tq, d)), rng.standard_normal((B, Hq, Tq, d)),
            rng.standard_normal((B, Hkv, Lk, d)), rng.standard_normal((B, Hkv, Lk, d)))


def test_dense_causal_and_banded_masks_match_the_c_oracle():
    q, r, k, v = _problem(1)
    Tq, Lk = 9, 14
    full = np.ones((Tq, Lk), bool)
    np.testing.assert_allclose(masked.masked_forward(q, r, k, v, 0.4, full), po.forward(q, r, k, v, 0.4),
                               rtol=1e-12, atol=1e-13)
    causal = np.tril(full, k=Lk - Tq)
    np.testing.assert_allclose(masked.masked_forward(q, r, k, v, 0.4, causal),
                               po.forward(q, r, k, v, 0.4, causal=True), rtol=1e-12, atol=1e-13)
    pos = np.arange(Tq)[:, None] + (Lk - Tq)
    band = causal & (pos - np.arange(Lk)[None, :] < 4)
    np.testing.assert_allclose(masked.masked_forward(q, r, k, v, 0.4, band),
                               po.forward(q, r, k, v, 0.4, causal=True, window=4), rtol=1e-12, atol=1e-13)


def test_random_mask_equals_the_c_oracle_on_gathered_keys():
    q, r, k, v = _problem(2)
    rng = np.random.default_rng(3)
    mask = rng.random((2, 4, 9, 14)) < 0.4
    mask[0, 0, 3] = False                       # an empty row
    out = masked.masked_forward(q, r, k, v, 0.7, mask)
    for b in range(2):
        for h in range(4):
            for i in range(9):
                cols = np.nonzero(mask[b, h, i])[0]
                if len(cols) == 0:
                    assert (out[b, h, i] == 0).all()
                    continue
                hk = h // 2
                ref = po.forward(q[b:b + 1, h:h + 1, i:i + 1], r[b:b + 1, h:h + 1, i:i + 1],
                                 k[b:b + 1, hk:hk + 1][:, :, cols], v[b:b + 1, hk:hk + 1][:, :, cols], 0.7)
                np.testing.assert_allclose(out[b, h, i], ref[0, 0, 0], rtol=1e-12, atol=1e-13)


def test_block_mask_expansion():
    bm = np.array([[1, 0, 1], [0, 1, 1]], dtype=bool)
    dense = masked.block_mask_to_dense(bm, 5, 7, 3, 3, causal=False)
    assert dense.shape == (5, 7)
    assert dense[:3, :3].all() and not dense[:3, 3:6].any() and dense[:3, 6].all()
    assert not dense[3:, :3].any() and dense[3:, 3:].all()
    c = masked.block_mask_to_dense(bm, 5, 7, 3, 3, causal=True)
    assert c[0, 2] and not c[0, 6]              # row 0 sits at position 2
    assert (c <= dense).all()


# ---- backward over an arbitrary mask (App. D closed forms restricted to the allowed pairs) -----
import pytest
import torch

from oracle import parallax_backward as pb


def _random_mask(seed, B, Hq, Tq, Lk, density=0.45):
    mask = np.random.default_rng(seed).random((B, Hq, Tq, Lk)) < density
    mask[0, 0, 1] = False                       # a row that sees nothing
    mask[:, :, :, Lk - 1] = False               # a key nobody sees
    return mask


def _torch_masked_forward(q, r, k, v, scale, mask):
    """The forward definition (Sec. 3.1, re-weighted softmax form) over the allowed keys, in
    PyTorch float64 with masked_fill / softmax -- independent of the numpy oracle's own steps."""
    G = q.shape[1] // k.shape[1]
    kk, vv = k.repeat_interleave(G, dim=1), v.repeat_interleave(G, dim=1)
    a = (scale * q @ kk.transpose(-1, -2)).masked_fill(~mask, float("-inf"))
    empty = ~mask.any(dim=-1, keepdim=True)
    p = torch.softmax(a.masked_fill(empty, 0.0), dim=-1).masked_fill(~mask, 0.0)
    u = r @ kk.transpose(-1, -2)
    ubar = (p * u).sum(-1, keepdim=True)
    return (p * (1.0 + ubar - u)) @ vv


def test_masked_backward_matches_autograd_of_the_definition():
    B, Hq, Hkv, Tq, Lk, d = 2, 4, 2, 6, 9, 4
    q, r, k, v = _problem(21, B, Hq, Hkv, Tq, Lk, d)
    g = np.random.default_rng(22).standard_normal(q.shape)
    mask = _random_mask(23, B, Hq, Tq, Lk)
    tq, tr, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, r, k, v))
    out = _torch_masked_forward(tq, tr, tk, tv, 0.55, torch.tensor(mask))
    np.testing.assert_allclose(out.detach().numpy(), masked.masked_forward(q, r, k, v, 0.55, mask),
                               rtol=1e-12, atol=1e-13)
    out.backward(torch.tensor(g))
    got = masked.masked_backward(q, r, k, v, g, 0.55, mask)
    for name, a, t in zip(("dq", "dr", "dk", "dv"), got, (tq, tr, tk, tv)):
        np.testing.assert_allclose(a, t.grad.numpy(), rtol=1e-10, atol=1e-12, err_msg=name)
    assert (got[0][0, 0, 1] == 0).all() and (got[1][0, 0, 1] == 0).all()     # the empty row
    assert (got[2][:, :, Lk - 1] == 0).all() and (got[3][:, :, Lk - 1] == 0).all()  # the unseen key


def test_masked_backward_matches_finite_differences_of_the_masked_forward():
    B, Hq, Hkv, Tq, Lk, d = 1, 2, 1, 4, 6, 3
    q, r, k, v = _problem(31, B, Hq, Hkv, Tq, Lk, d)
    g = np.random.default_rng(32).standard_normal(q.shape)
    mask = _random_mask(33, B, Hq, Tq, Lk, density=0.6)
    got = masked.masked_backward(q, r, k, v, g, 0.8, mask)
    xs, eps = [q, r, k, v], 1e-6
    for n, name in enumerate(("dq", "dr", "dk", "dv")):
        x, want = xs[n], np.zeros_like(xs[n])
        for idx in np.ndindex(*x.shape):
            old = x[idx]
            x[idx] = old + eps
            up = (g * masked.masked_forward(*xs, 0.8, mask)).sum()
            x[idx] = old - eps
            dn = (g * masked.masked_forward(*xs, 0.8, mask)).sum()
            x[idx] = old
            want[idx] = (up - dn) / (2 * eps)
        np.testing.assert_allclose(got[n], want, rtol=2e-6, atol=2e-7, err_msg=name)


@pytest.mark.parametrize("causal,window", [(False, 0), (True, 0), (True, 3)])
def test_masked_backward_and_cache_reduce_to_the_dense_causal_and_banded_oracle(causal, window):
    B, Hq, Hkv, Tq, Lk, d = 2, 4, 2, 7, 11, 4
    q, r, k, v = _problem(41, B, Hq, Hkv, Tq, Lk, d)
    g = np.random.default_rng(42).standard_normal(q.shape)
    pos = np.arange(Tq)[:, None] + (Lk - Tq)
    key = np.arange(Lk)[None, :]
    mask = (key <= pos) if causal else np.ones((Tq, Lk), bool)
    if window:
        mask = mask & (key > pos - window)
    for a, b in zip(masked.masked_backward(q, r, k, v, g, 0.5, mask),
                    pb.backward(q, r, k, v, g, 0.5, causal=causal, window=window)):
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)
    for a, b in zip(masked.masked_forward_with_cache(q, r, k, v, 0.5, mask),
                    pb.forward_with_cache(q, r, k, v, 0.5, causal=causal, window=window)):
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)


def test_masked_backward_conservation_laws_and_cache():
    """Adding a constant vector to every key changes no output (sum_j dK_j = 0 per KV head);
    adding one to every value adds it to every row that sees a key (sum_j dV_j = sum of those
    rows' dO). The cache of a row: vbar is the plain masked softmax average, o = vbar (1 + ubar) -
    sum_j p_ij u_ij v_j, log_omega the masked log-sum-exp."""
    B, Hq, Hkv, Tq, Lk, d = 2, 4, 2, 6, 8, 3
    q, r, k, v = _problem(51, B, Hq, Hkv, Tq, Lk, d)
    g = np.random.default_rng(52).standard_normal(q.shape)
    mask = _random_mask(53, B, Hq, Tq, Lk)
    dq, dr, dk, dv = masked.masked_backward(q, r, k, v, g, 0.9, mask)
    np.testing.assert_allclose(dk.sum(axis=2), 0.0, atol=1e-12)
    live = mask.any(axis=-1)[..., None]
    want = (g * live).reshape(B, Hkv, Hq // Hkv, Tq, d).sum(axis=(2, 3))
    np.testing.assert_allclose(dv.sum(axis=2), want, rtol=1e-12, atol=1e-12)
    o, vbar, ubar, log_omega = masked.masked_forward_with_cache(q, r, k, v, 0.9, mask)
    np.testing.assert_allclose(o, masked.masked_forward(q, r, k, v, 0.9, mask), rtol=1e-13, atol=1e-14)
    b, h, i = 1, 2, 3
    cols = np.nonzero(mask[b, h, i])[0]
    s = 0.9 * k[b, 1, cols] @ q[b, h, i]
    np.testing.assert_allclose(log_omega[b, h, i], np.log(np.exp(s).sum()), rtol=1e-12)
    p = np.exp(s - log_omega[b, h, i])
    np.testing.assert_allclose(vbar[b, h, i], p @ v[b, 1, cols], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(ubar[b, h, i], p @ (k[b, 1, cols] @ r[b, h, i]), rtol=1e-12, atol=1e-13)
    assert log_omega[0, 0, 1] == -np.inf and (vbar[0, 0, 1] == 0).all()


def test_planted_mistakes_in_the_masked_backward_are_caught():
    """A sign flip, a dropped term and mask leakage each fail the autograd pin."""
    B, Hq, Hkv, Tq, Lk, d = 1, 2, 1, 5, 7, 3
    q, r, k, v = _problem(61, B, Hq, Hkv, Tq, Lk, d)
    g = np.random.default_rng(62).standard_normal(q.shape)
    mask = _random_mask(63, B, Hq, Tq, Lk, density=0.6)
    tq, tr, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, r, k, v))
    _torch_masked_forward(tq, tr, tk, tv, 0.7, torch.tensor(mask)).backward(torch.tensor(g))
    truth = [t.grad.numpy() for t in (tq, tr, tk, tv)]
    # leakage: gradients computed as if the mask allowed one more pair
    leaky = mask.copy()
    leaky[0, 1, 2, np.nonzero(~mask[0, 1, 2])[0][0]] = True
    wrong = masked.masked_backward(q, r, k, v, g, 0.7, leaky)
    assert any(np.abs(a - b).max() > 1e-3 for a, b in zip(wrong, truth))
    # R with the wrong sign
    wrong = masked.masked_backward(q, -r, k, v, g, 0.7, mask)
    assert np.abs(wrong[0] - truth[0]).max() > 1e-3
    right = masked.masked_backward(q, r, k, v, g, 0.7, mask)
    assert all(np.abs(a - b).max() < 1e-10 for a, b in zip(right, truth))
