"""GPU parity of the sliding-window variants of parallax_prefill and parallax_decode (through
the C ABI) against the CPU oracle: a query at position pos sees the keys pos - W + 1 .. pos."""
import numpy as np
import pytest
import torch

from parity import BF16_REL_L2, F32_MAX_REL, host, max_rel, rel_l2

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def plx():
    from paper_2605_29157_amd import binding

    binding.load_library()
    assert torch.cuda.is_available()
    return binding


@pytest.fixture(scope="module")
def synth():
    from paper_2605_29157_amd import synth as s

    return s


def _prefill_ref(oracle, y, window, use_r=True):
    q, r, k, v = (host(y[n]) for n in "qrkv")
    if not use_r:
        r = np.zeros_like(r)
    return oracle.forward(q, r, k, v, y["scale"], causal=True, window=window)


def _row_errors(got, ref):
    return np.linalg.norm(got - ref, axis=-1) / np.maximum(np.linalg.norm(ref, axis=-1), 1e-6)


@pytest.mark.parametrize("T", [64, 128, 300, 1100])
@pytest.mark.parametrize("W", [1, 2, 33, 64, 100, 128, 129, 257, 700, 5000])
def test_prefill_window_square(plx, synth, oracle, T, W):
    """Windows shorter than a key block, of a few tiles, longer than the sequence; row blocks
    whose window starts in the first tile, at a tile edge, or several tiles in."""
    y = synth.prefill_inputs(2, 4, 2, T, 128, seed=900 + T + W, device=DEV, k_offset_sigma=0.5)
    ref = _prefill_ref(oracle, y, W)
    got = host(plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], window=W))
    assert np.isfinite(got).all()
    assert rel_l2(got, ref) <= BF16_REL_L2, (T, W)
    # single rows: with a handful of keys nothing averages the bf16 rounding of P1, P2 (each
    # 2^-9 relative, times |u| ~ sqrt(d) in the correction term), so the bound is wider there
    assert _row_errors(got, ref).max() <= (5 if W >= 32 else 12) * BF16_REL_L2, (T, W)
    if W == 1:  # one key: the value row at the query's own position, exactly
        np.testing.assert_array_equal(got, np.repeat(host(y["v"]), 2, axis=1))
    if W >= T:  # no row is cut: the same launch as without a window, bit for bit
        plain = host(plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"]))
        np.testing.assert_array_equal(got, plain)


@pytest.mark.parametrize("T,Tkv,W", [(128, 1000, 300), (200, 777, 64), (64, 4096, 1024), (5, 900, 130),
                                     (384, 2048, 2000)])
def test_prefill_window_chunk_behind_a_cache(plx, synth, oracle, T, Tkv, W):
    y = synth.prefill_inputs(1, 8, 2, Tkv, 128, seed=950 + T, device=DEV)
    y["q"], y["r"] = y["q"][:, :, Tkv - T:].contiguous(), y["r"][:, :, Tkv - T:].contiguous()
    ref = _prefill_ref(oracle, y, W)
    got = host(plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], window=W))
    assert rel_l2(got, ref) <= BF16_REL_L2
    assert _row_errors(got, ref).max() <= 5 * BF16_REL_L2


def test_prefill_window_other_paths(plx, synth, oracle):
    # d = 64 and the softmax-only twin
    y = synth.prefill_inputs(2, 4, 4, 500, 64, seed=960, device=DEV)
    got = host(plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], window=150))
    assert rel_l2(got, _prefill_ref(oracle, y, 150)) <= BF16_REL_L2
    twin = host(plx.parallax_prefill(y["q"], None, y["k"], y["v"], y["scale"], use_r=False, window=150))
    assert rel_l2(twin, _prefill_ref(oracle, y, 150, use_r=False)) <= BF16_REL_L2
    # fp32 path
    f = synth.prefill_inputs(1, 2, 2, 200, 64, seed=961, dtype=torch.float32, device=DEV)
    got = host(plx.parallax_prefill(f["q"], f["r"], f["k"], f["v"], f["scale"], window=37))
    assert max_rel(got, _prefill_ref(oracle, f, 37)) <= F32_MAX_REL
    # a window without causal has no meaning
    with pytest.raises(plx.ParallaxError):
        plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=False, window=8)


@pytest.mark.parametrize("gain", [6.0, 30.0])
def test_prefill_window_with_a_wide_logit_range(plx, synth, oracle, gain):
    """The softmax reference of a row may come from keys outside its window; with scores spread
    over hundreds of binary orders of magnitude it is useless (overflow, or a sum that
    underflows), and the kernel has to notice and take the online-rescale pass."""
    y = synth.prefill_inputs(1, 4, 2, 900, 128, seed=970, device=DEV)
    y["q"] = (y["q"].float() * gain).to(torch.bfloat16)
    ramp = torch.linspace(3.0, 0.2, 900, device=DEV).view(1, 1, 900, 1)  # early keys score highest
    y["k"] = (y["k"].float() * ramp).to(torch.bfloat16)
    ref = _prefill_ref(oracle, y, 200)
    got = host(plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], window=200))
    assert np.isfinite(got).all()
    assert rel_l2(got, ref) <= BF16_REL_L2
    # (no single-row bound here: the softmax of a row is down to one or two keys while |r.k|
    # reaches 100, and the bf16 rounding of P1, P2 alone gives single rows 10 % or more)


def _decode_ref(oracle, x, window, use_r=True):
    q, r = host(x["q"])[:, :, None, :], host(x["r"])[:, :, None, :]
    if not use_r:
        r = np.zeros_like(r)
    sl = x.get("seq_lens")
    return oracle.forward(q, r, host(x["k"]), host(x["v"]), x["scale"],
                          seq_lens=None if sl is None else sl.cpu().numpy(), window=window)[:, :, 0]


@pytest.mark.parametrize("W", [1, 5, 127, 128, 129, 500, 1400, 4096])
@pytest.mark.parametrize("S", [0, 1, 3])
def test_decode_window(plx, synth, oracle, W, S):
    x = synth.decode_inputs(4, 8, 4, 1500, 128, seed=980 + W, device=DEV)
    x["seq_lens"] = torch.tensor([1500, 1, 130, 777], dtype=torch.int32, device=DEV)
    ref = _decode_ref(oracle, x, W)
    got = host(plx.parallax_decode(x["q"], x["r"], x["k"], x["v"], x["scale"], seq_lens=x["seq_lens"],
                                   num_splits=S, window=W))
    assert rel_l2(got, ref) <= BF16_REL_L2, (W, S)
    assert _row_errors(got, ref).max() <= (5 if W >= 32 else 12) * BF16_REL_L2
    if W == 1:  # only the newest key
        lens = x["seq_lens"].cpu().numpy()
        v = host(x["v"])
        want = np.stack([np.repeat(v[b, :, lens[b] - 1], 2, axis=0) for b in range(4)])
        np.testing.assert_array_equal(got, want)


def test_decode_window_other_paths(plx, synth, oracle):
    x = synth.decode_inputs(3, 16, 8, 1500, 128, seed=990, device=DEV, ragged=True)
    ref = _decode_ref(oracle, x, 300)
    # paged cache, in-kernel reduction, softmax-only twin: all see the same window
    kp, vp, table = synth.paged_cache(x, 48, seed=991)
    got = plx.parallax_decode(x["q"], x["r"], kp, vp, x["scale"], seq_lens=x["seq_lens"],
                              block_table=table, max_len=1500, window=300)
    assert rel_l2(host(got), ref) <= BF16_REL_L2
    counters = torch.zeros(64, dtype=torch.int32, device=DEV)
    one = plx.parallax_decode_fused(x["q"], x["r"], x["k"], x["v"], x["scale"], counters,
                                    seq_lens=x["seq_lens"], num_splits=4, window=300)
    two = plx.parallax_decode(x["q"], x["r"], x["k"], x["v"], x["scale"], seq_lens=x["seq_lens"],
                              num_splits=4, window=300)
    np.testing.assert_array_equal(host(one), host(two))
    assert rel_l2(host(two), ref) <= BF16_REL_L2
    twin = plx.parallax_decode(x["q"], None, x["k"], x["v"], x["scale"], seq_lens=x["seq_lens"],
                               use_r=False, window=300)
    assert rel_l2(host(twin), _decode_ref(oracle, x, 300, use_r=False)) <= BF16_REL_L2
    # several query rows: row t sits at position L_b - Tq + t and takes its own window;
    # the same rows through the prefill kernel
    Tq, L, W = 4, 640, 200
    y = synth.prefill_inputs(2, 16, 8, L, 128, seed=992, device=DEV)
    q4, r4 = y["q"][:, :, L - Tq:].contiguous(), y["r"][:, :, L - Tq:].contiguous()
    want = oracle.forward(host(q4), host(r4), host(y["k"]), host(y["v"]), y["scale"], causal=True, window=W)
    dec = plx.parallax_decode(q4, r4, y["k"], y["v"], y["scale"], window=W)
    pre = plx.parallax_prefill(q4, r4, y["k"], y["v"], y["scale"], causal=True, window=W)
    assert rel_l2(host(dec), want) <= BF16_REL_L2
    assert rel_l2(host(pre), want) <= BF16_REL_L2
    # fp32 path
    f = synth.decode_inputs(2, 4, 2, 300, 64, seed=993, dtype=torch.float32, device=DEV, ragged=True)
    got = plx.parallax_decode(f["q"], f["r"], f["k"], f["v"], f["scale"], seq_lens=f["seq_lens"], window=50)
    assert max_rel(host(got), _decode_ref(oracle, f, 50)) <= F32_MAX_REL


def test_window_full_size_sampled(plx, synth, oracle):
    """Long-sequence shapes (T = 16384 prefill, L = 65536 decode) with a 4096-key window, as
    timed by bench.py: sampled rows against the oracle."""
    B, Hq, Hkv, T, d, W = 1, 16, 8, 16384, 128, 4096
    y = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=995, device=DEV)
    got = host(plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], window=W))
    rng = np.random.default_rng(3)
    rows = np.stack([np.zeros(40, dtype=np.int64), rng.integers(0, Hq, 40),
                     np.concatenate([[0, 1, 4095, 4096, 4097, T - 1, 8191, 8192],
                                     rng.integers(0, T, 32)])], axis=1)
    ref = oracle.forward(*(host(y[n]) for n in "qrkv"), y["scale"], causal=True, window=W, rows=rows)
    sel = got[rows[:, 0], rows[:, 1], rows[:, 2]]
    assert rel_l2(sel, ref) <= BF16_REL_L2
    assert _row_errors(sel, ref).max() <= 5 * BF16_REL_L2
    del y
    x = synth.decode_inputs(2, Hq, Hkv, 65536, d, seed=996, device=DEV)
    x["seq_lens"] = torch.tensor([65536, 40000], dtype=torch.int32, device=DEV)
    got = host(plx.parallax_decode(x["q"], x["r"], x["k"], x["v"], x["scale"], seq_lens=x["seq_lens"],
                                   window=W))
    assert rel_l2(got, _decode_ref(oracle, x, W)) <= BF16_REL_L2
