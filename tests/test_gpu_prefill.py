"""GPU parity of parallax_prefill (through the C ABI) against the CPU oracle."""
import numpy as np
import pytest
import torch

from parity import BF16_REL_L2, F32_MAX_REL, host, max_rel, oracle_prefill, rel_l2

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


def _run(plx, y, **kw):
    out = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], **kw)
    torch.cuda.synchronize()
    return host(out)


def test_config1_tiny_causal_fp32(plx, synth, oracle):
    """benchmark configuration 1: B=1, 2 heads (no GQA), T=128, d=64, fp32, scale 1/8."""
    y = synth.prefill_inputs(1, 2, 2, 128, 64, seed=1001, dtype=torch.float32, device=DEV)
    assert abs(y["scale"] - 0.125) < 1e-12
    ref = oracle_prefill(oracle, y)
    got = _run(plx, y)
    assert max_rel(got, ref) <= F32_MAX_REL
    # row 0 sees exactly key 0
    np.testing.assert_allclose(got[0, :, 0], host(y["v"])[0, :, 0], rtol=1e-6, atol=1e-6)
    # element-wise relative error where the output is not near a zero crossing
    rms = np.sqrt((ref ** 2).mean())
    el = np.abs(got - ref) / np.maximum(np.abs(ref), 1e-2 * rms)
    assert el.max() <= 1e-3


@pytest.mark.parametrize("T", [1, 31, 32, 33, 64, 65, 127, 128, 129, 300, 513])
@pytest.mark.parametrize("causal", [True, False])
def test_small_lengths_bf16(plx, synth, oracle, T, causal):
    y = synth.prefill_inputs(2, 4, 2, T, 128, seed=300 + T, device=DEV, k_offset_sigma=0.5)
    ref = oracle_prefill(oracle, y, causal=causal)
    got = _run(plx, y, causal=causal)
    assert np.isfinite(got).all()
    assert rel_l2(got, ref) <= BF16_REL_L2, (T, causal)
    if causal:  # row 0 = v_0 exactly
        np.testing.assert_array_equal(got[:, :, 0], np.repeat(host(y["v"])[:, :, 0], 2, axis=1))


def test_softmax_only_twin(plx, synth, oracle):
    y = synth.prefill_inputs(1, 4, 2, 400, 128, seed=401, device=DEV)
    ref = oracle_prefill(oracle, y, use_r=False)
    assert rel_l2(_run(plx, y, use_r=False), ref) <= BF16_REL_L2
    # and a zero probe through the Parallax kernel gives the same thing
    y0 = dict(y)
    y0["r"] = torch.zeros_like(y["r"])
    assert rel_l2(_run(plx, y0), ref) <= BF16_REL_L2


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("gain", [12.0, 40.0])
def test_large_logit_range_takes_the_safe_path(plx, synth, oracle, gain, causal):
    """Scores spread over hundreds of binary orders of magnitude: a fixed softmax reference from
    the first key block overflows, so the kernel must fall back to the online max/rescale pass
    (a plain exp without max subtraction would give inf/NaN here)."""
    y = synth.prefill_inputs(1, 4, 2, 700, 128, seed=811, device=DEV)
    y["q"] = (y["q"].float() * gain).to(torch.bfloat16)
    # make late keys much more attractive than early ones for half of the rows
    ramp = torch.linspace(0.2, 3.0, 700, device=DEV).view(1, 1, 700, 1)
    y["k"] = (y["k"].float() * ramp).to(torch.bfloat16)
    ref = oracle_prefill(oracle, y, causal=causal)
    got = _run(plx, y, causal=causal)
    assert np.isfinite(got).all()
    assert rel_l2(got, ref) <= BF16_REL_L2


@pytest.mark.parametrize("T,Tkv,causal,window", [(1, 1, True, 0), (31, 31, True, 0), (255, 255, True, 0),
                                                   (256, 256, True, 0), (257, 257, True, 0), (300, 300, False, 0),
                                                   (513, 513, True, 0), (1100, 1100, True, 0), (200, 777, True, 0),
                                                   (5, 600, True, 0), (130, 515, False, 0), (700, 700, True, 1),
                                                   (700, 700, True, 40), (520, 1500, True, 300)])
def test_head_dim_64_two_row_sub_blocks_per_wave(plx, synth, oracle, T, Tkv, causal, window):
    """d = 64 runs 64 query rows per wave (256 per workgroup): lengths around and far from
    multiples of 256, chunks behind a cache, windows, the softmax-only twin, the online-rescale
    pass, and the row cache written by the same kernel family."""
    from oracle import parallax_backward as pb

    y = synth.prefill_inputs(2, 4, 2, Tkv, 64, seed=860 + T + window, device=DEV, k_offset_sigma=0.5)
    y["q"], y["r"] = y["q"][:, :, Tkv - T:].contiguous(), y["r"][:, :, Tkv - T:].contiguous()
    q, r, k, v = (host(y[n]) for n in "qrkv")
    ref = oracle.forward(q, r, k, v, y["scale"], causal=causal, window=window)
    got = host(plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=causal, window=window))
    assert rel_l2(got, ref) <= BF16_REL_L2
    ref0 = oracle.forward(q, np.zeros_like(r), k, v, y["scale"], causal=causal, window=window)
    got0 = host(plx.parallax_prefill(y["q"], None, y["k"], y["v"], y["scale"], causal=causal, window=window, use_r=False))
    assert rel_l2(got0, ref0) <= BF16_REL_L2
    # row cache: same output bits, vbar / ubar / log-sum-exp against the definition
    o, vbar, stats = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=causal, window=window,
                                          save_for_backward=True)
    np.testing.assert_array_equal(host(o), got)
    _, vb, ub, lw = pb.forward_with_cache(q, r, k, v, y["scale"], causal=causal, window=window)
    assert rel_l2(host(vbar), vb) <= BF16_REL_L2
    np.testing.assert_allclose(host(stats)[..., 0], lw * 1.4426950408889634, rtol=0, atol=2e-2)
    assert np.linalg.norm(host(stats)[..., 1] - ub) <= BF16_REL_L2 * np.linalg.norm(ub) + 1e-6
    # scores spread over hundreds of binades: the fixed reference overflows, the online pass takes over
    if window == 0:
        big = dict(y)
        big["q"] = (y["q"].float() * 30.0).to(torch.bfloat16)
        big["k"] = (y["k"].float() * torch.linspace(0.2, 3.0, Tkv, device=DEV).view(1, 1, Tkv, 1)).to(torch.bfloat16)
        refb = oracle.forward(host(big["q"]), r, host(big["k"]), v, y["scale"], causal=causal)
        gotb = host(plx.parallax_prefill(big["q"], y["r"], big["k"], y["v"], y["scale"], causal=causal))
        assert np.isfinite(gotb).all()
        assert rel_l2(gotb, refb) <= BF16_REL_L2


def test_scale_zero_is_uniform_weighting(plx, synth, oracle):
    """scale = 0 is the wide-bandwidth limit (uniform softmax weights)."""
    y = synth.prefill_inputs(1, 4, 2, 260, 128, seed=821, device=DEV, r_scale=0.2)
    y["scale"] = 0.0
    ref = oracle_prefill(oracle, y)
    assert rel_l2(_run(plx, y), ref) <= BF16_REL_L2


@pytest.mark.parametrize("Hq,Hkv,d", [(2, 2, 128), (8, 2, 128), (4, 2, 64), (16, 8, 64), (16, 1, 128), (24, 2, 64)])
def test_head_layouts(plx, synth, oracle, Hq, Hkv, d):
    y = synth.prefill_inputs(1, Hq, Hkv, 333, d, seed=500 + Hq + d, device=DEV)
    ref = oracle_prefill(oracle, y)
    assert rel_l2(_run(plx, y), ref) <= BF16_REL_L2


def test_strided_inputs(plx, synth, oracle):
    """[B, T, H, d] storage passed as permuted views."""
    y = synth.prefill_inputs(2, 4, 2, 200, 128, seed=601, device=DEV)
    ref = oracle_prefill(oracle, y)
    ys = dict(y)
    for n in "qrkv":
        ys[n] = y[n].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert rel_l2(_run(plx, ys), ref) <= BF16_REL_L2


def test_prefill_last_row_equals_decode(plx, synth):
    """The last causal row sees every key: it must agree with a decode step over the same cache
    (two different kernels, same operator)."""
    y = synth.prefill_inputs(2, 16, 8, 1024, 128, seed=701, device=DEV)
    pre = _run(plx, y)[:, :, -1, :]
    dec = plx.parallax_decode(y["q"][:, :, -1, :].contiguous(), y["r"][:, :, -1, :].contiguous(),
                              y["k"], y["v"], y["scale"])
    torch.cuda.synchronize()
    assert rel_l2(host(dec), pre.astype(np.float64)) <= BF16_REL_L2


def _chunk(y, T):
    """The last T query rows of a square problem over all its keys."""
    c = dict(y)
    c["q"], c["r"] = y["q"][:, :, -T:].contiguous(), y["r"][:, :, -T:].contiguous()
    return c


@pytest.mark.parametrize("T,Tkv", [(1, 1), (1, 300), (5, 69), (64, 64 + 37), (128, 1000), (130, 515),
                                   (257, 2048), (100, 100 + 64), (31, 4096)])
@pytest.mark.parametrize("causal", [True, False])
def test_chunked_prefill_bf16(plx, synth, oracle, T, Tkv, causal):
    """T query rows over Tkv >= T keys: causal rows are the last T positions of the sequence."""
    y = _chunk(synth.prefill_inputs(2, 4, 2, Tkv, 128, seed=800 + T + Tkv, device=DEV,
                                    k_offset_sigma=0.5), T)
    ref = oracle_prefill(oracle, y, causal=causal)
    got = _run(plx, y, causal=causal)
    assert got.shape == ref.shape and np.isfinite(got).all()
    assert rel_l2(got, ref) <= BF16_REL_L2, (T, Tkv, causal)
    # per-row check: a wrong diagonal offset shows up in single rows long before the total
    row_err = np.linalg.norm(got - ref, axis=-1) / np.maximum(np.linalg.norm(ref, axis=-1), 1e-6)
    assert row_err.max() <= 5 * BF16_REL_L2, (T, Tkv, causal, int(row_err.argmax()))


def test_chunked_prefill_matches_square_tail_and_decode(plx, synth):
    """Same kernel, two launches: the chunk equals the tail rows of the square problem; a
    one-row chunk equals a decode step over the cache."""
    y = synth.prefill_inputs(2, 16, 8, 1536, 128, seed=811, device=DEV)
    square = _run(plx, y)
    for T in (1, 200):
        c = _chunk(y, T)
        got = _run(plx, c)
        assert rel_l2(got, square[:, :, -T:].astype(np.float64)) <= BF16_REL_L2
    dec = plx.parallax_decode(y["q"][:, :, -1].contiguous(), y["r"][:, :, -1].contiguous(),
                              y["k"], y["v"], y["scale"])
    torch.cuda.synchronize()
    assert rel_l2(host(dec), _run(plx, _chunk(y, 1))[:, :, 0].astype(np.float64)) <= BF16_REL_L2


def test_chunked_prefill_fp32_and_d64(plx, synth, oracle):
    y = _chunk(synth.prefill_inputs(1, 2, 2, 200, 64, seed=812, dtype=torch.float32, device=DEV), 50)
    assert max_rel(_run(plx, y), oracle_prefill(oracle, y)) <= F32_MAX_REL
    y = _chunk(synth.prefill_inputs(2, 4, 4, 333, 64, seed=813, device=DEV), 77)
    assert rel_l2(_run(plx, y), oracle_prefill(oracle, y)) <= BF16_REL_L2
    with pytest.raises(plx.ParallaxError):  # causal needs at least as many keys as rows
        bad = dict(y)
        bad["k"], bad["v"] = y["k"][:, :, :50].contiguous(), y["v"][:, :, :50].contiguous()
        _run(plx, bad)


def _sample_rows(B, Hq, T, n_random, seed, tile=128, edge_batches=2):
    """Row sample of a large prefill: on EVERY head of the first `edge_batches` batch entries the
    rows 0..127, the last 128 and every 128-row boundary - 1, +0, +1; one random row of every
    128-row block of every (batch, head), so that each workgroup of the launch has a compared
    row; and n_random rows drawn uniformly."""
    rng = np.random.default_rng(seed)
    rows = set()
    for b in range(min(edge_batches, B)):
        for h in range(Hq):
            for i in list(range(0, min(tile, T))) + list(range(max(T - tile, 0), T)):
                rows.add((b, h, i))
            for edge in range(tile, T, tile):
                for i in (edge - 1, edge, edge + 1):
                    if 0 <= i < T:
                        rows.add((b, h, i))
    for b in range(B):
        for h in range(Hq):
            for blk in range(0, T, tile):
                rows.add((b, h, int(rng.integers(blk, min(blk + tile, T)))))
    for _ in range(n_random):
        rows.add((int(rng.integers(B)), int(rng.integers(Hq)), int(rng.integers(T))))
    return np.array(sorted(rows), dtype=np.int32)


def test_config4_prefill_bf16_sampled(plx, synth, oracle):
    """benchmark configuration 4: B=4, T=4096, 16/8 heads, d=128, keys offset per (b, kv head) by
    N(0, 0.5^2), the launch bench.py times; oracle on about 15 000 sampled rows: first and last
    128 rows and every 128-row boundary +- 1 on all heads of two batch entries, a row of every
    workgroup, 2048 random rows. Bound over the sample and per row."""
    y = synth.prefill_inputs(4, 16, 8, 4096, 128, seed=1004, device=DEV, k_offset_sigma=0.5)
    got = _run(plx, y)
    assert np.isfinite(got).all()
    rows = _sample_rows(4, 16, 4096, 2048, seed=4)
    assert len(rows) >= 2 * 16 * (256 + 3 * 31) + 2048
    ref = oracle_prefill(oracle, y, rows=rows)
    sub = got[rows[:, 0], rows[:, 1], rows[:, 2]]
    assert rel_l2(sub, ref) <= BF16_REL_L2
    per_row = np.linalg.norm(sub - ref, axis=1) / np.linalg.norm(ref, axis=1)
    assert per_row.max() <= 5e-2, rows[int(per_row.argmax())]


def test_config5a_long_prefill_sampled(plx, synth, oracle):
    """Config 5 part one: B=2, T=16384, probe scaled by 0.1."""
    y = synth.prefill_inputs(2, 16, 8, 16384, 128, seed=1005, device=DEV, r_scale=0.1)
    got = _run(plx, y)
    assert np.isfinite(got).all()
    rows = _sample_rows(2, 16, 16384, 300, seed=5, edge_batches=0)
    ref = oracle_prefill(oracle, y, rows=rows)
    sub = got[rows[:, 0], rows[:, 1], rows[:, 2]]
    assert rel_l2(sub, ref) <= BF16_REL_L2


def test_register_only_mfma_loop_runs_and_counts_its_flops(plx):
    """The matrix-rate ceiling kernel: every lane ends with a finite, non-trivial sum, and the
    sustained rate is of the order of the chip's (between a tenth of and the nominal peak)."""
    sink = torch.zeros(256 * 256, dtype=torch.float32, device=DEV)
    plx.parallax_util_mfma(256, 50, sink)          # warm-up
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    flops = plx.parallax_util_mfma(256, 5000, sink)
    e1.record()
    torch.cuda.synchronize()
    s = sink.cpu().numpy()
    assert np.isfinite(s).all() and np.abs(s).max() > 1.0 and len(np.unique(s)) > 1000
    rate = flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    assert 250.0 < rate < 2600.0, rate
