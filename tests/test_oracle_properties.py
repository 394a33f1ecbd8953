"""Property tests of the oracle over random small problems (CPU): the identities of the pin
suite hold for every shape, scale and head grouping hypothesis comes up with."""
import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import forms


def _draw(rng, B, Hq, Hkv, Tq, Lk, d):
    f = lambda *sh: rng.standard_normal(sh)
    return f(B, Hq, Tq, d), f(B, Hq, Tq, d), f(B, Hkv, Lk, d), f(B, Hkv, Lk, d)


shapes = st.tuples(st.integers(1, 2), st.sampled_from([(1, 1), (2, 1), (4, 2), (3, 3)]),
                   st.integers(1, 6), st.integers(0, 7), st.integers(1, 6),
                   st.floats(0.0, 1.5), st.integers(0, 2 ** 31 - 1))


@settings(max_examples=40, deadline=None)
@given(shapes, st.booleans())
def test_forms_weights_and_invariances(oracle, shape, causal):
    B, (Hq, Hkv), Tq, extra, d, scale, seed = shape
    Lk = Tq + extra
    rng = np.random.default_rng(seed)
    q, r, k, v = _draw(rng, B, Hq, Hkv, Tq, Lk, d)
    out = oracle.forward(q, r, k, v, scale, causal=causal)
    # the covariance form and the fold over keys with odd groupings and split points agree
    np.testing.assert_allclose(forms.covariance_form(q, r, k, v, scale, causal=causal), out,
                               rtol=1e-9, atol=1e-9)
    cuts = sorted(set(int(c) for c in rng.integers(0, Lk + 1, size=2)))
    np.testing.assert_allclose(
        forms.streaming_form(q, r, k, v, scale, causal=causal, tile=3, row_block=2, split_points=cuts),
        out, rtol=1e-9, atol=1e-9)
    # key translation leaves the output unchanged; values enter affinely (weights sum to one)
    c = rng.standard_normal(d)
    np.testing.assert_allclose(oracle.forward(q, r, k + c, v, scale, causal=causal), out,
                               rtol=1e-8, atol=1e-8)
    A, bvec = rng.standard_normal((d, d)), rng.standard_normal(d)
    np.testing.assert_allclose(oracle.forward(q, r, k, v @ A + bvec, scale, causal=causal),
                               out @ A + bvec, rtol=1e-8, atol=1e-8)
    # zero probe: plain softmax attention of the same rows
    zero = oracle.forward(q, np.zeros_like(r), k, v, scale, causal=causal)
    G = Hq // Hkv
    for b in range(B):
        for h in range(Hq):
            for i in range(Tq):
                n = i + 1 + (Lk - Tq) if causal else Lk
                a = scale * (k[b, h // G, :n] @ q[b, h, i])
                w = np.exp(a - a.max())
                np.testing.assert_allclose(zero[b, h, i], (w / w.sum()) @ v[b, h // G, :n],
                                           rtol=1e-10, atol=1e-10)
