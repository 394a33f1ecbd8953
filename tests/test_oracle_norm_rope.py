"""Pins of the RMSNorm + RoPE oracle (oracle/norm_rope.py) against things that are not itself."""
import numpy as np
import pytest

from oracle import norm_rope as nr


def test_hand_worked_rotation_in_two_dimensions():
    # d = 2: one pair, frequency theta^0 = 1, so the angle is the position itself
    x = np.array([[1.0, 0.0], [0.0, 2.0], [3.0, 4.0]])
    out = nr.rope(x, np.array([np.pi / 2, np.pi, 0.5]), theta=1.0e6)
    np.testing.assert_allclose(out[0], [0.0, 1.0], atol=1e-15)
    np.testing.assert_allclose(out[1], [0.0, -2.0], atol=1e-15)
    np.testing.assert_allclose(out[2], [3 * np.cos(0.5) - 4 * np.sin(0.5), 3 * np.sin(0.5) + 4 * np.cos(0.5)],
                               atol=1e-15)


def test_frequencies_follow_theta_to_the_minus_2i_over_d():
    # a one-hot pair at index i rotates by pos * theta^(-2i/d): read the angle back
    d, theta, pos = 8, 100.0, 3.0
    for i in range(d // 2):
        x = np.zeros((1, d))
        x[0, 2 * i] = 1.0
        out = nr.rope(x, np.array([pos]), theta=theta)[0]
        ang = np.arctan2(out[2 * i + 1], out[2 * i])
        want = pos * theta ** (-2.0 * i / d)
        assert abs((ang - want + np.pi) % (2 * np.pi) - np.pi) < 1e-12
        assert np.count_nonzero(np.abs(out) > 1e-15) <= 2


def test_rms_norm_properties():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((3, 5, 16)) * 7.0
    y = nr.rms_norm(x, np.ones(16), eps=0.0)
    np.testing.assert_allclose((y * y).mean(-1), 1.0, atol=1e-12)          # unit RMS
    np.testing.assert_allclose(nr.rms_norm(13.0 * x, np.ones(16), eps=0.0), y, atol=1e-12)  # scale free
    gamma = rng.standard_normal(16)
    np.testing.assert_allclose(nr.rms_norm(x, gamma, eps=0.0), y * gamma, atol=1e-12)
    # eps enters under the root, next to the mean square
    one = np.full((1, 4), 2.0)
    np.testing.assert_allclose(nr.rms_norm(one, np.ones(4), eps=5.0), one / 3.0, atol=1e-15)


def test_rope_is_an_isometry_identity_at_zero_and_positions_add():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((2, 3, 6, 32))
    pos = np.arange(6) + 40
    y = nr.rope(x, pos)
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)
    np.testing.assert_array_equal(nr.rope(x, np.zeros(6)), x)
    np.testing.assert_allclose(nr.rope(nr.rope(x, pos), 7 * np.ones(6)), nr.rope(x, pos + 7), atol=1e-11)


def test_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(3)
    q, k = rng.standard_normal((1, 32)), rng.standard_normal((1, 32))
    for m, n in [(5, 2), (100, 97), (4003, 4000)]:
        s = nr.rope(q, np.array([m])) @ nr.rope(k, np.array([n])).T
        np.testing.assert_allclose(s, nr.rope(q, np.array([3])) @ k.T, rtol=1e-9, atol=1e-9)
    # ... and do change with it
    a = nr.rope(q, np.array([3])) @ k.T
    b = nr.rope(q, np.array([4])) @ k.T
    assert abs(a - b).max() > 1e-3


@pytest.mark.parametrize("mistake", ["rotate_half_pairs", "sign", "freq_exponent", "norm_after_rope_weight"])
def test_planted_mistakes_are_rejected(mistake):
    """Plausible mistakes, written out here, must differ from the oracle on a generic input."""
    rng = np.random.default_rng(4)
    x = rng.standard_normal((4, 16))
    pos = np.array([1.0, 2.0, 3.0, 50.0])
    gamma = rng.standard_normal(16)
    good = nr.norm_rope(x, gamma, pos, theta=1.0e4)
    d = 16
    freq = 1.0e4 ** (-np.arange(0, d, 2) / d)
    y = x / np.sqrt((x * x).mean(-1, keepdims=True) + 1e-6) * gamma
    if mistake == "rotate_half_pairs":      # pairs (i, i + d/2) instead of adjacent ones
        ang = pos[:, None] * freq
        wrong = np.concatenate([y[:, :8] * np.cos(ang) - y[:, 8:] * np.sin(ang),
                                y[:, :8] * np.sin(ang) + y[:, 8:] * np.cos(ang)], axis=1)
    elif mistake == "sign":
        wrong = nr.rope(y, -pos, theta=1.0e4)
    elif mistake == "freq_exponent":        # theta^(-i/d)
        ang = pos[:, None] * 1.0e4 ** (-np.arange(0, d // 2) / d)
        wrong = np.empty_like(y)
        wrong[:, 0::2] = y[:, 0::2] * np.cos(ang) - y[:, 1::2] * np.sin(ang)
        wrong[:, 1::2] = y[:, 0::2] * np.sin(ang) + y[:, 1::2] * np.cos(ang)
    else:                                   # weight applied after the rotation
        wrong = nr.rope(x / np.sqrt((x * x).mean(-1, keepdims=True) + 1e-6), pos, theta=1.0e4) * gamma
    assert np.abs(wrong - good).max() > 1e-3
