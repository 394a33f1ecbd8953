"""Pins of the MLA-style decode oracle (oracle/mla.py) against things that are not itself."""
import numpy as np
import torch

from oracle import mla
from oracle import parallax_oracle as po


def _problem(seed, B=2, Hq=5, L=9, dc=6, dr=2):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, Hq, dc + dr))
    r = 0.5 * rng.standard_normal((B, Hq, dc + dr))
    ckv = rng.standard_normal((B, L, dc + dr))
    return q, r, ckv


def test_equals_the_forward_oracle_on_one_shared_head_with_zero_padded_values():
    """One KV head shared by all query heads, keys = the whole row, values = the latent part
    padded with zeros to the key width: the C oracle then computes the same sums (the padded
    output dimensions come out as zeros)."""
    dc, dr = 6, 2
    q, r, ckv = _problem(1, dc=dc, dr=dr)
    lens = np.array([9, 4], dtype=np.int32)
    got = mla.mla_decode(q, r, ckv, dc, 0.4, lens)
    vpad = ckv.copy()
    vpad[..., dc:] = 0.0
    ref = po.forward(q[:, :, None, :], r[:, :, None, :], ckv[:, None], vpad[:, None], 0.4, causal=False,
                     seq_lens=lens)[:, :, 0]
    np.testing.assert_allclose(got, ref[..., :dc], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(ref[..., dc:], 0.0, atol=1e-15)


def test_zero_probe_is_library_softmax_attention_with_a_narrower_value():
    dc, dr = 8, 4
    q, r, ckv = _problem(2, B=1, Hq=3, L=11, dc=dc, dr=dr)
    got = mla.mla_decode(q, np.zeros_like(r), ckv, dc, 0.3)
    tq = torch.tensor(q)[:, :, None, :]                       # [B, H, 1, dk]
    tk = torch.tensor(ckv)[:, None].expand(1, 3, 11, dc + dr)
    tv = tk[..., :dc]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=0.3)[:, :, 0].numpy()
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_two_tokens_closed_form():
    """o = vbar - p (1 - p) (v_1 - v_2) <k_1 - k_2, rho> with p the weight of token 1."""
    dc, dr = 3, 2
    q, r, ckv = _problem(3, B=1, Hq=2, L=2, dc=dc, dr=dr)
    got = mla.mla_decode(q, r, ckv, dc, 0.7)
    k1, k2 = ckv[0, 0], ckv[0, 1]
    for h in range(2):
        a = 0.7 * np.array([k1 @ q[0, h], k2 @ q[0, h]])
        p = 1.0 / (1.0 + np.exp(a[1] - a[0]))
        vbar = p * k1[:dc] + (1 - p) * k2[:dc]
        want = vbar - p * (1 - p) * (k1[:dc] - k2[:dc]) * ((k1 - k2) @ r[0, h])
        np.testing.assert_allclose(got[0, h], want, rtol=1e-12, atol=1e-13)


def test_common_shift_of_the_rope_part_changes_nothing_and_empty_sequences_give_zeros():
    dc, dr = 5, 3
    q, r, ckv = _problem(4, dc=dc, dr=dr)
    base = mla.mla_decode(q, r, ckv, dc, 0.5)
    shifted = ckv.copy()
    shifted[..., dc:] += np.array([0.3, -1.1, 2.0])            # every key moves by the same vector
    np.testing.assert_allclose(mla.mla_decode(q, r, shifted, dc, 0.5), base, rtol=1e-10, atol=1e-12)
    out = mla.mla_decode(q, r, ckv, dc, 0.5, np.array([0, 3]))
    assert (out[0] == 0).all() and np.abs(out[1]).max() > 0


def test_planted_mistakes_are_rejected():
    import inspect

    src = inspect.getsource(mla)
    mutants = {
        "value_takes_the_rope_part": ("values = ckv[b, :n, :d_latent]", "values = ckv[b, :n, -d_latent:]"),
        "score_on_the_latent_only": ("a = scale * (keys @ q[b, h])", "a = scale * (keys[:, :d_latent] @ q[b, h, :d_latent])"),
        "probe_on_the_latent_only": ("u = keys @ r[b, h]", "u = keys[:, :d_latent] @ r[b, h, :d_latent]"),
        "probe_sign": ("(1.0 + ubar - u)", "(1.0 - ubar + u)"),
        "probe_scaled": ("u = keys @ r[b, h]", "u = scale * (keys @ r[b, h])"),
    }
    dc = 6
    q, r, ckv = _problem(5, dc=dc, dr=2)
    vpad = ckv.copy()
    vpad[..., dc:] = 0.0
    ref = po.forward(q[:, :, None, :], r[:, :, None, :], ckv[:, None], vpad[:, None], 0.4,
                     causal=False)[:, :, 0, :dc]
    for name, (old, new) in mutants.items():
        assert src.count(old) == 1, name
        ns = {}
        exec(compile(src.replace(old, new), "<mutant>", "exec"), ns)
        got = ns["mla_decode"](q, r, ckv, dc, 0.4)
        assert np.abs(got - ref).max() > 1e-6, "no pin noticed the planted mistake '%s'" % name
