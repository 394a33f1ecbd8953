"""Pins for the CPU oracle: facts the paper and the mathematics fix, none of which come from
the oracle itself or from the HIP path. Each test says which mistake it would catch."""
import os

import numpy as np
import pytest
import torch

from oracle import forms

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def _problem(B=2, Hq=4, Hkv=2, T=9, d=5, seed=0):
    return (_rand((B, Hq, T, d), seed), _rand((B, Hq, T, d), seed + 1),
            _rand((B, Hkv, T, d), seed + 2), _rand((B, Hkv, T, d), seed + 3))


# ---- hand-worked values -------------------------------------------------------------------
def test_hand_worked_two_key_example(oracle):
    """Sec. 3.1 forward equation on numbers worked by hand (sign of the correction, which
    operand the probe multiplies)."""
    rows = np.loadtxt(os.path.join(GOLD, "two_key_example.txt"))
    for row in rows:
        q = row[0:2].reshape(1, 1, 1, 2)
        k = row[2:6].reshape(1, 1, 2, 2)
        v = np.stack([row[6:8], np.zeros(2)], axis=1).reshape(1, 1, 2, 2)
        rho = row[8:10].reshape(1, 1, 1, 2)
        out = oracle.forward(q, rho, k, v, row[10])
        assert abs(out[0, 0, 0, 0] - row[11]) < 1e-14
        assert out[0, 0, 0, 1] == 0.0


# ---- P1: brute force with explicit weight matrices (Sec. 4.4, s_ij) -----------------------
def _brute(q, r, k, v, scale, causal, seq_lens=None, window=0):
    B, Hq, Tq, d = q.shape
    _, Hkv, Lk, _ = k.shape
    G = Hq // Hkv
    out = np.zeros_like(q)
    W = np.zeros((B, Hq, Tq, Lk))
    for b in range(B):
        for h in range(Hq):
            K, V = k[b, h // G], v[b, h // G]
            A = scale * q[b, h] @ K.T
            mask = np.ones((Tq, Lk), dtype=bool)
            if causal:
                mask = np.tril(mask, k=Lk - Tq)  # row i is position i + Lk - Tq
            elif seq_lens is not None:
                mask[:, seq_lens[b]:] = False
            if window:  # position of row i minus key position < window
                n_b = Lk if causal or seq_lens is None else int(seq_lens[b])
                pos = np.arange(Tq)[:, None] + (n_b - Tq)
                mask &= pos - np.arange(Lk)[None, :] < window
            A = np.where(mask, A, -np.inf)
            P = np.exp(A - A.max(axis=1, keepdims=True))
            P = P / P.sum(axis=1, keepdims=True)
            U = r[b, h] @ K.T
            ubar = (P * U).sum(axis=1, keepdims=True)
            S = P * (1.0 + ubar - U)
            W[b, h] = S
            out[b, h] = S @ V
    return out, W


@pytest.mark.parametrize("causal", [True, False])
def test_brute_force_weight_matrix(oracle, causal):
    q, r, k, v = _problem(seed=10)
    ref, W = _brute(q, r, k, v, 0.37, causal)
    out = oracle.forward(q, r, k, v, 0.37, causal=causal)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-12)
    # the Parallax weights of a row sum to one and may be negative (Sec. 4.4)
    np.testing.assert_allclose(W.sum(axis=-1), 1.0, atol=1e-12)
    assert (W < 0).any()


def test_chunked_causal_is_the_tail_of_the_square_case(oracle):
    """Tq query rows over Lk > Tq keys with the causal flag: the queries are the last Tq
    positions, so the result is the last Tq rows of the square causal problem (pinned above),
    a one-row chunk is plain decode over all keys, and a top-left aligned mask is wrong."""
    from oracle import forms

    B, Hq, Hkv, L, d, Tq = 2, 4, 2, 13, 5, 4
    q, r = _rand((B, Hq, L, d), 31), _rand((B, Hq, L, d), 32)
    k, v = _rand((B, Hkv, L, d), 33), _rand((B, Hkv, L, d), 34)
    square = oracle.forward(q, r, k, v, 0.41, causal=True)
    qc, rc = q[:, :, L - Tq:], r[:, :, L - Tq:]
    chunk = oracle.forward(qc, rc, k, v, 0.41, causal=True)
    np.testing.assert_allclose(chunk, square[:, :, L - Tq:], rtol=1e-14, atol=1e-14)
    ref, W = _brute(qc, rc, k, v, 0.41, True)
    np.testing.assert_allclose(chunk, ref, rtol=1e-12, atol=1e-12)
    assert (W[:, :, 0, L - Tq + 1:] == 0).all() and (W[:, :, 0, :L - Tq + 1] != 0).all()
    # top-left alignment (row i sees keys <= i) is a different, wrong, result
    topleft = np.stack([oracle.forward(qc[:, :, i:i + 1], rc[:, :, i:i + 1], k[:, :, :i + 1],
                                       v[:, :, :i + 1], 0.41)[:, :, 0] for i in range(Tq)], axis=2)
    assert np.abs(topleft - chunk).max() > 1e-3
    # one query row: decode over all L keys
    one = oracle.forward(q[:, :, L - 1:], r[:, :, L - 1:], k, v, 0.41, causal=True)
    np.testing.assert_allclose(one, oracle.forward(q[:, :, L - 1:], r[:, :, L - 1:], k, v, 0.41),
                               rtol=1e-14, atol=1e-14)
    # the covariance and streaming forms take the same alignment
    np.testing.assert_allclose(forms.covariance_form(qc, rc, k, v, 0.41, causal=True), chunk,
                               rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(forms.streaming_form(qc, rc, k, v, 0.41, causal=True, tile=4,
                                                    row_block=3, split_points=[5, 9]), chunk,
                               rtol=1e-10, atol=1e-10)
    with pytest.raises(ValueError):
        oracle.forward(q, r, k[:, :, :L - 1], v[:, :, :L - 1], 0.41, causal=True)  # Tq > Lk


@pytest.mark.parametrize("window", [1, 2, 3, 5, 12, 13, 40])
def test_sliding_window_brute_force_and_special_cases(oracle, window):
    """Sliding window (the usual definition: a query at position pos sees positions
    pos - W + 1 .. pos): explicit band mask; W = 1 returns the value row at the query's own
    position; W >= the sequence is no window; a windowed row equals the unwindowed problem on
    the slice of keys it sees; decode rows take the window from their own length."""
    B, Hq, Hkv, L, d, Tq = 2, 4, 2, 13, 5, 6
    q, r = _rand((B, Hq, Tq, d), 41), _rand((B, Hq, Tq, d), 42)
    k, v = _rand((B, Hkv, L, d), 43), _rand((B, Hkv, L, d), 44)
    out = oracle.forward(q, r, k, v, 0.43, causal=True, window=window)
    ref, W = _brute(q, r, k, v, 0.43, True, window=window)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-12)
    # exactly min(window, position + 1) non-zero weights per row, ending on the diagonal
    for i in range(Tq):
        pos = i + L - Tq
        nz = np.nonzero(W[0, 0, i])[0]
        assert nz.max() == pos and nz.min() == max(0, pos - window + 1)
    if window == 1:
        np.testing.assert_allclose(out, np.repeat(v[:, :, L - Tq:], 2, axis=1), atol=1e-14)
    if window >= L:
        np.testing.assert_array_equal(out, oracle.forward(q, r, k, v, 0.43, causal=True))
    # row i alone, over exactly the keys it sees, with no mask at all
    i = 3
    pos = i + L - Tq
    lo = max(0, pos - window + 1)
    alone = oracle.forward(q[:, :, i:i + 1], r[:, :, i:i + 1], k[:, :, lo:pos + 1], v[:, :, lo:pos + 1], 0.43)
    np.testing.assert_allclose(out[:, :, i:i + 1], alone, rtol=1e-13, atol=1e-13)
    # decode: one query row per sequence at position len_b - 1
    lens = np.array([13, 4], dtype=np.int32)
    dec = oracle.forward(q[:, :, :1], r[:, :, :1], k, v, 0.43, seq_lens=lens, window=window)
    refd, Wd = _brute(q[:, :, :1], r[:, :, :1], k, v, 0.43, False, lens, window=window)
    np.testing.assert_allclose(dec, refd, rtol=1e-12, atol=1e-12)
    assert np.count_nonzero(Wd[1, 0, 0]) == min(window, 4)
    # several rows without a position (not causal) have no window
    with pytest.raises(ValueError):
        oracle.forward(q, r, k, v, 0.43, window=window)


def test_brute_force_ragged_decode_and_gqa(oracle):
    """Decode shape (one query row), ragged lengths, GQA mapping h -> h // G."""
    B, Hq, Hkv, L, d = 3, 6, 2, 17, 4
    q, r = _rand((B, Hq, 1, d), 1), _rand((B, Hq, 1, d), 2)
    k, v = _rand((B, Hkv, L, d), 3), _rand((B, Hkv, L, d), 4)
    lens = np.array([17, 1, 9], dtype=np.int32)
    ref, _ = _brute(q, r, k, v, 0.5, False, lens)
    out = oracle.forward(q, r, k, v, 0.5, seq_lens=lens)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-12)
    # a wrong head mapping (h % Hkv instead of h // G) must be visible on this input
    wrong = oracle.forward(q, r, k[:, [0, 1, 0, 1, 0, 1]], v[:, [0, 1, 0, 1, 0, 1]], 0.5,
                           seq_lens=lens)
    assert np.abs(wrong - ref).max() > 1e-3


def test_row_list_matches_full(oracle):
    q, r, k, v = _problem(seed=20)
    full = oracle.forward(q, r, k, v, 0.3, causal=True)
    rows = np.array([[0, 0, 0], [1, 3, 8], [0, 2, 4], [1, 1, 7]], dtype=np.int32)
    sub = oracle.forward(q, r, k, v, 0.3, causal=True, rows=rows)
    for n, (b, h, i) in enumerate(rows):
        np.testing.assert_array_equal(sub[n], full[b, h, i])
    # float32 containers are widened exactly
    q32, r32, k32, v32 = (x.astype(np.float32) for x in (q, r, k, v))
    a = oracle.forward(q32, r32, k32, v32, 0.3, causal=True)
    bb = oracle.forward(*(x.astype(np.float64) for x in (q32, r32, k32, v32)), 0.3, causal=True)
    np.testing.assert_allclose(a, bb, rtol=1e-14, atol=1e-14)
    sub32 = oracle.forward(q32, r32, k32, v32, 0.3, causal=True, rows=rows)
    for n, (b, h, i) in enumerate(rows):
        np.testing.assert_allclose(sub32[n], a[b, h, i], rtol=1e-14, atol=1e-14)


# ---- P2: R = 0 gives softmax attention (Sec. 3.2 strong-regularisation limit) -------------
@pytest.mark.parametrize("causal", [True, False])
def test_zero_probe_is_library_softmax_attention(oracle, causal):
    q, r, k, v = _problem(B=2, Hq=4, Hkv=2, T=11, d=8, seed=30)
    out = oracle.forward(q, np.zeros_like(r), k, v, 0.25, causal=causal)
    tq, tk, tv = (torch.from_numpy(x) for x in (q, k, v))
    tk = tk.repeat_interleave(2, dim=1)
    tv = tv.repeat_interleave(2, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=causal,
                                                           scale=0.25).numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-11, atol=1e-12)


# ---- P3: affine equivariance in V (weights sum to one) ------------------------------------
def test_affine_equivariance_in_values(oracle):
    q, r, k, v = _problem(seed=40)
    A = _rand((5, 5), 41)
    bvec = _rand((5,), 42)
    base = oracle.forward(q, r, k, v, 0.4, causal=True)
    moved = oracle.forward(q, r, k, v @ A + bvec, 0.4, causal=True)
    np.testing.assert_allclose(moved, base @ A + bvec, rtol=1e-10, atol=1e-10)
    const = oracle.forward(q, r, k, np.broadcast_to(bvec, v.shape).copy(), 0.4, causal=True)
    np.testing.assert_allclose(const, np.broadcast_to(bvec, q.shape), rtol=1e-12, atol=1e-12)


# ---- P4: key-translation invariance (softmax shift + centred probe score) -----------------
def test_key_translation_invariance(oracle):
    q, r, k, v = _problem(seed=50)
    c = _rand((5,), 51, scale=3.0)
    base = oracle.forward(q, r, k, v, 0.4, causal=True)
    moved = oracle.forward(q, r, k + c, v, 0.4, causal=True)
    np.testing.assert_allclose(moved, base, rtol=1e-9, atol=1e-9)
    # a version that forgets to centre u (o = sum p (1 - u) v) is NOT invariant: make sure the
    # input would expose it
    _, Hkv, _, _ = k.shape
    P_u = np.einsum("bhid,bhjd->bhij", r, np.repeat(k + c, 2, axis=1))
    assert np.abs(P_u).max() > 1.0


# ---- P5: three forms agree (Sec. 3.1 both sides; Sec. 3.3 expanded/streaming form) --------
@pytest.mark.parametrize("causal", [True, False])
def test_three_forms_agree(oracle, causal):
    q, r, k, v = _problem(B=1, Hq=4, Hkv=2, T=23, d=6, seed=60)
    scale = 0.45
    a = oracle.forward(q, r, k, v, scale, causal=causal)
    b = forms.covariance_form(q, r, k, v, scale, causal=causal)
    np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-10)
    for tile, rb, cuts in [(4, 3, None), (7, 8, [5, 5, 16]), (32, 23, [1]), (1, 1, [22])]:
        c = forms.streaming_form(q, r, k, v, scale, causal=causal, tile=tile, row_block=rb,
                                 split_points=cuts)
        np.testing.assert_allclose(a, c, rtol=1e-9, atol=1e-9)


# ---- P6: scale = 0 (h -> inf) closed form via running means (Sec. 3.2) --------------------
def test_wide_bandwidth_limit_closed_form(oracle):
    q, r, k, v = _problem(B=1, Hq=2, Hkv=2, T=12, d=4, seed=70)
    out = oracle.forward(q, r, k, v, 0.0, causal=True)
    n = np.arange(1, 13)[None, None, :, None]
    vbar = np.cumsum(v, axis=2) / n
    kbar = np.cumsum(k, axis=2) / n
    S = np.cumsum(np.einsum("bhtv,bhtk->bhtvk", v, k), axis=2) / n[..., None]
    S_tilde = S - np.einsum("bhtv,bhtk->bhtvk", vbar, kbar)
    ref = vbar - np.einsum("bhtvk,bhtk->bhtv", S_tilde, r)
    np.testing.assert_allclose(out, ref, rtol=1e-11, atol=1e-11)


# ---- P7: one key, two keys ----------------------------------------------------------------
def test_one_and_two_key_closed_forms(oracle):
    d = 6
    q, rho = _rand((1, 1, 1, d), 80), _rand((1, 1, 1, d), 81)
    k, v = _rand((1, 1, 2, d), 82), _rand((1, 1, 2, d), 83)
    scale = 0.7
    one = oracle.forward(q, rho, k[:, :, :1], v[:, :, :1], scale)
    np.testing.assert_allclose(one[0, 0, 0], v[0, 0, 0], rtol=0, atol=1e-15)
    a = scale * (k[0, 0] @ q[0, 0, 0])
    p = 1.0 / (1.0 + np.exp(a[1] - a[0]))  # weight of key 0
    vbar = p * v[0, 0, 0] + (1 - p) * v[0, 0, 1]
    ref = vbar - p * (1 - p) * (v[0, 0, 0] - v[0, 0, 1]) * ((k[0, 0, 0] - k[0, 0, 1]) @ rho[0, 0, 0])
    two = oracle.forward(q, rho, k, v, scale)
    np.testing.assert_allclose(two[0, 0, 0], ref, rtol=1e-12, atol=1e-13)
    # causal row 0 sees exactly key 0 (diagonal included)
    qq, rr = _rand((1, 1, 2, d), 84), _rand((1, 1, 2, d), 85)
    c = oracle.forward(qq, rr, k, v, scale, causal=True)
    np.testing.assert_allclose(c[0, 0, 0], v[0, 0, 0], rtol=0, atol=1e-15)


# ---- P8: values affine in keys ------------------------------------------------------------
def test_values_affine_in_keys(oracle):
    d, L = 5, 14
    q, rho = _rand((1, 1, 1, d), 90), _rand((1, 1, 1, d), 91)
    k = _rand((1, 1, L, d), 92)
    A, bvec = _rand((d, d), 93), _rand((d,), 94)
    v = k @ A.T + bvec
    scale = 0.6
    out = oracle.forward(q, rho, k, v, scale)[0, 0, 0]
    a = scale * (k[0, 0] @ q[0, 0, 0])
    p = np.exp(a - a.max())
    p /= p.sum()
    kbar = p @ k[0, 0]
    var_k = (k[0, 0] - kbar).T @ (p[:, None] * (k[0, 0] - kbar))
    ref = A @ (kbar - var_k @ rho[0, 0, 0]) + bvec
    np.testing.assert_allclose(out, ref, rtol=1e-11, atol=1e-11)


# ---- P9: exact local-linear attention identity (Sec. 2.1 LLA forward, Sec. 3.1 reformulation)
def test_lla_identity_with_solved_probe(oracle):
    d, L, lam, h = 4, 10, 0.3, 1.7
    q = _rand((d,), 100, 0.5)
    k = _rand((L, d), 101)
    v = _rand((L, d), 102)
    w = np.exp(k @ q / h)
    z = k - q
    omega = w.sum()
    mu = w @ z
    Sigma = z.T @ (w[:, None] * z) + lam * np.eye(d)
    rho_star = np.linalg.solve(Sigma, mu)
    o_lla = ((w * (1 - z @ rho_star)) @ v) / (omega - mu @ rho_star)
    p = w / omega
    o_sa = p @ v
    tbar = p @ (z @ rho_star)
    assert 0.0 <= tbar < 1.0  # Prop. 1
    eta = tbar / (1 - tbar)
    o_plx = oracle.forward(q.reshape(1, 1, 1, d), rho_star.reshape(1, 1, 1, d),
                           k.reshape(1, 1, L, d), v.reshape(1, 1, L, d), 1.0 / h)[0, 0, 0]
    np.testing.assert_allclose(o_lla - o_sa, (1 + eta) * (o_plx - o_sa), rtol=1e-9, atol=1e-12)


# ---- P10: split-merge associativity incl. empty parts (App. C) -----------------------------
def test_split_merge_associativity():
    q, r, k, v = _problem(B=1, Hq=2, Hkv=1, T=19, d=4, seed=110)
    Q, R, K, V = q[0, 0, -3:], r[0, 0, -3:], k[0, 0], v[0, 0]
    whole = forms.streaming_partial(Q, R, K, V, 0.5, 5, 0, 19)
    ref = forms.finalize(whole)
    for cuts in ([0, 19], [0, 0, 7, 7, 19], [0, 1, 2, 18, 19, 19]):
        parts = [forms.streaming_partial(Q, R, K, V, 0.5, 3, cuts[i], cuts[i + 1])
                 for i in range(len(cuts) - 1)]
        np.testing.assert_allclose(forms.finalize(forms.merge_partials(parts)), ref,
                                   rtol=1e-11, atol=1e-12)
    # merging is order independent
    parts = [forms.streaming_partial(Q, R, K, V, 0.5, 4, a, b) for a, b in [(0, 6), (6, 13), (13, 19)]]
    np.testing.assert_allclose(forms.finalize(forms.merge_partials(parts[::-1])), ref,
                               rtol=1e-11, atol=1e-12)


def test_empty_key_set_is_zero(oracle):
    """Undefined in the paper (empty softmax); the documented reading is a zero row."""
    q, r = _rand((2, 2, 1, 4), 120), _rand((2, 2, 1, 4), 121)
    k, v = _rand((2, 1, 5, 4), 122), _rand((2, 1, 5, 4), 123)
    out = oracle.forward(q, r, k, v, 1.0, seq_lens=np.array([0, 5], dtype=np.int32))
    assert np.all(out[0] == 0.0) and np.abs(out[1]).max() > 0
