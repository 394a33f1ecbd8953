"""Seeded random valid shapes through the C ABI against the oracle: layouts, lengths, GQA groups,
head dims, chunk sizes, page sizes and split counts in combinations the hand-picked cases miss."""
import numpy as np
import pytest
import torch

from parity import BF16_REL_L2, host, oracle_decode, oracle_prefill, rel_l2

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def plx():
    from paper_2605_29157_amd import binding

    binding.load_library()
    return binding


@pytest.fixture(scope="module")
def synth():
    from paper_2605_29157_amd import synth as s

    return s


def _heads(rng):
    G = int(rng.choice([1, 2, 4, 8]))
    Hkv = int(rng.choice([1, 2, 3]))
    return G * Hkv, Hkv


@pytest.mark.parametrize("case", range(24))
def test_random_prefill_shapes(plx, synth, oracle, case):
    rng = np.random.default_rng(9000 + case)
    Hq, Hkv = _heads(rng)
    d = int(rng.choice([64, 128]))
    B = int(rng.integers(1, 3))
    T = int(rng.choice([1, 2, 31, 33, 64, 65, 127, 128, 129, 191, 200, 256, 300, 385]))
    extra = int(rng.choice([0, 0, 1, 17, 63, 64, 100, 129, 500]))
    causal = bool(rng.integers(0, 2))
    use_r = bool(rng.integers(0, 4))  # mostly with the probe
    y = synth.prefill_inputs(B, Hq, Hkv, T + extra, d, seed=9100 + case, device=DEV,
                             k_offset_sigma=float(rng.choice([0.0, 0.5])),
                             r_scale=float(rng.choice([1.0, 0.1])))
    y["q"], y["r"] = y["q"][:, :, extra:].contiguous(), y["r"][:, :, extra:].contiguous()
    scale = y["scale"] * float(rng.choice([1.0, 0.25, 2.0]))
    yy = dict(y, scale=scale)
    ref = oracle_prefill(oracle, yy, causal=causal, use_r=use_r)
    out = plx.parallax_prefill(y["q"], y["r"] if use_r else None, y["k"], y["v"], scale,
                               causal=causal, use_r=use_r)
    torch.cuda.synchronize()
    got = host(out)
    assert np.isfinite(got).all()
    assert rel_l2(got, ref) <= BF16_REL_L2, (B, Hq, Hkv, T, extra, d, causal, use_r)


@pytest.mark.parametrize("case", range(24))
def test_random_decode_shapes(plx, synth, oracle, case):
    rng = np.random.default_rng(9500 + case)
    Hq, Hkv = _heads(rng)
    d = int(rng.choice([64, 128]))
    B = int(rng.integers(1, 6))
    L = int(rng.choice([1, 5, 127, 128, 129, 500, 1024, 1500, 3001]))
    ragged = bool(rng.integers(0, 2))
    use_r = bool(rng.integers(0, 4))
    n_bt = (L + 127) // 128
    S = int(rng.choice([0, 1, 2, 3, 7, 16])) if n_bt > 1 else int(rng.choice([0, 1]))
    x = synth.decode_inputs(B, Hq, Hkv, L, d, seed=9600 + case, device=DEV, ragged=ragged,
                            r_scale=float(rng.choice([1.0, 0.1])))
    ref = oracle_decode(oracle, x, use_r=use_r)
    kw = dict(seq_lens=x.get("seq_lens"), use_r=use_r, num_splits=S)
    out = plx.parallax_decode(x["q"], x["r"] if use_r else None, x["k"], x["v"], x["scale"], **kw)
    torch.cuda.synchronize()
    got = host(out)
    assert rel_l2(got, ref) <= BF16_REL_L2, (B, Hq, Hkv, L, d, ragged, use_r, S)
    # the same cache behind a block table gives the same bits
    page = int(rng.choice([1, 7, 16, 64, 100, 256]))
    kp, vp, table = synth.paged_cache(x, page, seed=9700 + case)
    paged = plx.parallax_decode(x["q"], x["r"] if use_r else None, kp, vp, x["scale"],
                                block_table=table, max_len=L, **kw)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(paged), got)
