"""Seeded random valid shapes through the C ABI against the oracle: layouts, lengths, GQA groups,
head dims, chunk sizes, page sizes and split counts in combinations the hand-picked cases miss."""
import numpy as np
import pytest
import torch

from parity import BF16_REL_L2, assert_gradient_close, host, oracle_decode, oracle_prefill, rel_l2

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


@pytest.mark.parametrize("case", range(20))
def test_random_backward_shapes_with_and_without_window(plx, synth, case):
    """Forward with row cache + backward on random shapes against the float64 closed forms;
    half of the causal cases under a sliding window of random width."""
    from oracle import parallax_backward as pb

    rng = np.random.default_rng(9800 + case)
    Hq, Hkv = _heads(rng)
    d = int(rng.choice([64, 128]))
    B = int(rng.integers(1, 3))
    T = int(rng.choice([2, 33, 64, 65, 127, 128, 129, 191, 200, 256, 300, 385, 520]))
    extra = int(rng.choice([0, 0, 1, 17, 63, 64, 100, 129, 400]))
    causal = bool(rng.integers(0, 4))   # mostly causal
    window = int(rng.choice([0, 3, 40, 64, 65, 128, 200, 333])) if causal else 0
    y = synth.prefill_inputs(B, Hq, Hkv, T + extra, d, seed=9850 + case, device=DEV,
                             r_scale=float(rng.choice([1.0, 0.3])))
    y["q"], y["r"] = y["q"][:, :, extra:].contiguous(), y["r"][:, :, extra:].contiguous()
    g = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=9851 + case, device=DEV)["q"].contiguous()
    o, vbar, stats = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=causal,
                                          save_for_backward=True, window=window)
    grads = plx.parallax_prefill_backward(y["q"], y["r"], y["k"], y["v"], o, vbar, stats, g, y["scale"],
                                          causal=causal, window=window)
    torch.cuda.synchronize()
    want = pb.backward(*(host(y[n]) for n in "qrkv"), host(g), y["scale"], causal=causal, window=window)
    for name, got, ref in zip(("dq", "dr", "dk", "dv"), grads, want):
        assert_gradient_close(name, host(got), ref, BF16_REL_L2, (B, Hq, Hkv, T, extra, d, causal, window))


@pytest.mark.parametrize("case", range(16))
def test_random_block_masks_and_windows_forward(plx, synth, oracle, case):
    """Random block masks (per batch / per head / shared) and random windows on random shapes."""
    from oracle import masked

    rng = np.random.default_rng(9900 + case)
    Hq, Hkv = _heads(rng)
    d = int(rng.choice([64, 128]))
    B = int(rng.integers(1, 3))
    T = int(rng.choice([1, 64, 100, 128, 129, 300, 700, 1100]))
    extra = int(rng.choice([0, 0, 5, 64, 130, 900]))
    causal = bool(rng.integers(0, 3))
    y = synth.prefill_inputs(B, Hq, Hkv, T + extra, d, seed=9950 + case, device=DEV)
    y["q"], y["r"] = y["q"][:, :, extra:].contiguous(), y["r"][:, :, extra:].contiguous()
    q, r, k, v = (host(y[n]) for n in "qrkv")
    nrb, nkt = -(-T // 128), -(-(T + extra) // 64)
    lead = [(), (Hq,), (B, 1), (B, Hq)][int(rng.integers(0, 4))]
    bm = rng.random(lead + (nrb, nkt)) < float(rng.choice([0.15, 0.5, 0.9]))
    out = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=causal,
                               block_mask=torch.as_tensor(bm, device=DEV))
    torch.cuda.synchronize()
    bm4 = bm.reshape((1,) * (4 - bm.ndim) + bm.shape)   # missing leading dims are shared
    dense = masked.block_mask_to_dense(bm4, T, T + extra, 128, 64, causal)
    ref = masked.masked_forward(q, r, k, v, y["scale"], dense)
    got = host(out)
    assert np.isfinite(got).all()
    assert np.linalg.norm(got - ref) <= BF16_REL_L2 * np.linalg.norm(ref) + 1e-6, (B, Hq, Hkv, T, extra, d, causal, lead)
    if causal:
        W = int(rng.choice([1, 5, 64, 100, 129, 500]))
        outw = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=True, window=W)
        torch.cuda.synchronize()
        refw = oracle.forward(q, r, k, v, y["scale"], causal=True, window=W)
        assert rel_l2(host(outw), refw) <= BF16_REL_L2, (T, extra, d, W)
