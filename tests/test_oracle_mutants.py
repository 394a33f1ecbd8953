"""The pins must be able to fail: plant plausible mistakes in a COPY of the oracle's C source
(on the CPU, in a temp dir), and check that the pinned facts reject every mutant."""
import functools
import os
import subprocess

import numpy as np
import pytest

from oracle import parallax_oracle as po

MUTANTS = {
    "sign_of_correction": ("(1.0 + ubar - u[j])", "(1.0 - ubar + u[j])"),
    "uncentred_probe": ("(1.0 + ubar - u[j])", "(1.0 - u[j])"),
    "probe_scaled_like_q": ("u[j] = s2;", "u[j] = scale * s2;"),
    "probe_uses_q": ("s2 += rho[c] * kj[c];", "s2 += q[c] * kj[c];"),
    "ubar_unweighted": ("ubar += a[j] * u[j];", "ubar += u[j] / (double)n_keys;"),
    "causal_excludes_diagonal": ("n_keys = (int64_t)i + 1 + (Lk - Tq);",
                                 "n_keys = (int64_t)i + (Lk - Tq);"),
    "causal_chunk_top_left_aligned": ("n_keys = (int64_t)i + 1 + (Lk - Tq);",
                                      "n_keys = (int64_t)i + 1;"),
    "window_one_key_too_many": ("n_keys > window) ? n_keys - window : 0;",
                                "n_keys > window) ? n_keys - window - 1 : 0;"),
    "window_counted_from_the_start": ("kb + first * d, vb + first * d, n_keys - first,",
                                      "kb, vb, n_keys - first,"),
    "gqa_modulo": ("const int hk = h / G;", "const int hk = h % Hkv;"),
    "no_max_subtraction_no_norm": ("a[j] /= omega;", "a[j] /= 1.0;"),
}


def _pins(fwd):
    """A compact subset of the pins; returns the names of those that FAIL."""
    failed = []
    rng = np.random.default_rng(5)
    # hand-worked example (tests/golden/two_key_example.txt)
    q = np.zeros((1, 1, 1, 2))
    k = np.array([[[[1.0, 0.0], [-1.0, 0.0]]]])
    v = np.array([[[[1.0, 0.0], [3.0, 0.0]]]])
    if abs(fwd(q, np.array([[[[1.0, 0.0]]]]), k, v, 1.0)[0, 0, 0, 0] - 3.0) > 1e-12:
        failed.append("hand")
    # two-key closed form with scale != 1
    d = 4
    q, rho = rng.standard_normal((1, 1, 1, d)), rng.standard_normal((1, 1, 1, d))
    k, v = rng.standard_normal((1, 1, 2, d)), rng.standard_normal((1, 1, 2, d))
    a = 0.7 * (k[0, 0] @ q[0, 0, 0])
    p = 1.0 / (1.0 + np.exp(a[1] - a[0]))
    ref = p * v[0, 0, 0] + (1 - p) * v[0, 0, 1] - p * (1 - p) * (v[0, 0, 0] - v[0, 0, 1]) * (
        (k[0, 0, 0] - k[0, 0, 1]) @ rho[0, 0, 0])
    if np.abs(fwd(q, rho, k, v, 0.7)[0, 0, 0] - ref).max() > 1e-10:
        failed.append("two_key")
    # key-translation invariance, causal row 0 = v_0, constant values, GQA order
    B, Hq, Hkv, T = 1, 4, 2, 7
    q, r = rng.standard_normal((B, Hq, T, d)), rng.standard_normal((B, Hq, T, d))
    k, v = rng.standard_normal((B, Hkv, T, d)), rng.standard_normal((B, Hkv, T, d))
    base = fwd(q, r, k, v, 0.5, causal=True)
    if np.abs(fwd(q, r, k + 2.0, v, 0.5, causal=True) - base).max() > 1e-8:
        failed.append("translation")
    if np.abs(base[0, :, 0] - np.repeat(v[0, :, 0], 2, axis=0)).max() > 1e-12:
        failed.append("row0")
    if np.abs(fwd(q, r, k, np.ones_like(v), 0.5, causal=True) - 1.0).max() > 1e-10:
        failed.append("constant_values")
    # causal chunk of one query row over T keys = that row with every key allowed
    one = fwd(q[:, :, -1:], r[:, :, -1:], k, v, 0.5, causal=True)
    if np.abs(one - fwd(q[:, :, -1:], r[:, :, -1:], k, v, 0.5)).max() > 1e-12:
        failed.append("chunk_alignment")
    # sliding window of one position returns the value row at the query's own position, and a
    # window of two is the two-key closed form on the last two allowed keys
    w1 = fwd(q, r, k, v, 0.5, causal=True, window=1)
    if np.abs(w1 - np.repeat(v, 2, axis=1)).max() > 1e-12:
        failed.append("window_one")
    w2 = fwd(q[:, :1, -1:], r[:, :1, -1:], k[:, :1], v[:, :1], 0.5, causal=True, window=2)[0, 0, 0]
    k2, v2 = k[0, 0, -2:], v[0, 0, -2:]
    a = 0.5 * (k2 @ q[0, 0, -1])
    p = 1.0 / (1.0 + np.exp(a[1] - a[0]))
    ref = p * v2[0] + (1 - p) * v2[1] - p * (1 - p) * (v2[0] - v2[1]) * ((k2[0] - k2[1]) @ r[0, 0, -1])
    if np.abs(w2 - ref).max() > 1e-10:
        failed.append("window_two")
    return failed


def test_unmutated_source_passes_compact_pins():
    assert _pins(po.forward) == []


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_rejected(name, tmp_path):
    old, new = MUTANTS[name]
    src = open(os.path.join(os.path.dirname(po.__file__), "parallax_oracle.c")).read()
    assert src.count(old) >= 1, "mutation site vanished from the oracle source"
    cfile = tmp_path / "mutant.c"
    cfile.write_text(src.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-o",
                           str(lib), str(cfile), "-lm"])
    fwd = functools.partial(po.forward, _lib_override=po._bind(str(lib)))
    assert _pins(fwd) != [], "no pin noticed the planted mistake '%s'" % name
