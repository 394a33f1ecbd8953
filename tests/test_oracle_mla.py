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


def _mutate(fn, old, new):
    import inspect

    src = inspect.getsource(fn)
    assert src.count(old) == 1, old
    ns = {"np": np}
    exec(compile(src.replace(old, new), "<mutant>", "exec"), ns)
    return ns[fn.__name__]


def test_planted_mistakes_are_rejected():
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
        got = _mutate(mla.mla_decode, old, new)(q, r, ckv, dc, 0.4)
        assert np.abs(got - ref).max() > 1e-6, "no pin noticed the planted mistake '%s'" % name


def test_planted_mistakes_in_the_several_row_form_are_rejected():
    mutants = {
        "row_position_off_by_one": ("pos = n - Tq + t", "pos = n - Tq + t + 1"),
        "rows_at_the_first_positions": ("pos = n - Tq + t", "pos = t"),
        "window_one_too_wide": ("first = max(0, pos - window + 1)", "first = max(0, pos - window)"),
        "window_ignored": ("first = max(0, pos - window + 1) if window > 0 else 0", "first = 0"),
        "value_takes_the_rope_part": ("values = keys[:, :d_latent]", "values = keys[:, -d_latent:]"),
        "probe_sign": ("(1.0 + ubar - u)", "(1.0 - ubar + u)"),
        "same_query_row_for_all": ("a = scale * (keys @ q[b, h, t])", "a = scale * (keys @ q[b, h, 0])"),
    }
    dc = 6
    q, r, ckv = _rows_problem(6, B=1, Hq=2, Tq=3, L=9, dc=dc, dr=2)
    vpad = ckv.copy()
    vpad[..., dc:] = 0.0
    ref = po.forward(q, r, ckv[:, None], vpad[:, None], 0.4, causal=True, window=4)[..., :dc]
    np.testing.assert_allclose(mla.mla_rows(q, r, ckv, dc, 0.4, window=4), ref, rtol=1e-12, atol=1e-13)
    for name, (old, new) in mutants.items():
        got = _mutate(mla.mla_rows, old, new)(q, r, ckv[:, :9], dc, 0.4, None, 4)
        assert got.shape == ref.shape
        assert np.abs(got - ref).max() > 1e-6, "no pin noticed the planted mistake '%s'" % name


def _rows_problem(seed, B=2, Hq=3, Tq=4, L=10, dc=6, dr=2):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, Hq, Tq, dc + dr))
    r = 0.5 * rng.standard_normal((B, Hq, Tq, dc + dr))
    ckv = rng.standard_normal((B, L, dc + dr))
    return q, r, ckv


def test_several_rows_and_window_equal_the_forward_oracle_on_one_shared_head():
    """Causal / sliding-window attention of the C oracle over one shared KV head whose values are
    the latent part padded with zeros: rows at the last Tq positions, ragged lengths."""
    dc, dr = 6, 2
    q, r, ckv = _rows_problem(11, dc=dc, dr=dr)
    vpad = ckv.copy()
    vpad[..., dc:] = 0.0
    lens = np.array([10, 7], dtype=np.int32)
    for window in (0, 1, 3, 50):
        got = mla.mla_rows(q, r, ckv, dc, 0.45, lens, window=window)
        for b in range(2):                      # (the C oracle takes one key count per call)
            n = int(lens[b])
            ref = po.forward(q[b:b + 1], r[b:b + 1], ckv[b:b + 1, None, :n], vpad[b:b + 1, None, :n], 0.45,
                             causal=True, window=window)
            np.testing.assert_allclose(got[b], ref[0, ..., :dc], rtol=1e-12, atol=1e-13)


def test_rows_reduce_to_single_row_decode_and_rows_before_the_sequence_are_zero():
    dc = 5
    q, r, ckv = _rows_problem(12, B=2, Hq=2, Tq=3, L=8, dc=dc, dr=3)
    lens = np.array([8, 2], dtype=np.int32)     # second sequence: shorter than Tq
    got = mla.mla_rows(q, r, ckv, dc, 0.6, lens)
    for b in range(2):
        for t in range(3):
            n_seen = int(lens[b]) - 3 + t + 1
            if n_seen <= 0:
                assert (got[b, :, t] == 0).all()
                continue
            one = mla.mla_decode(q[b:b + 1, :, t], r[b:b + 1, :, t], ckv[b:b + 1], dc, 0.6, np.array([n_seen]))
            np.testing.assert_allclose(got[b, :, t], one[0], rtol=1e-13, atol=1e-14)
    # a window of one token: the output is that token's latent part (p = 1, u = ubar)
    w1 = mla.mla_rows(q, r, ckv, dc, 0.6, np.array([8, 8]), window=1)
    for t in range(3):
        np.testing.assert_allclose(w1[:, :, t], np.broadcast_to(ckv[:, None, 8 - 3 + t, :dc], w1[:, :, t].shape),
                                   rtol=1e-13, atol=1e-14)
