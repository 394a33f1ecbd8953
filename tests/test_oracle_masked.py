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
