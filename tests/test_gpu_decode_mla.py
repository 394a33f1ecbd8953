"""GPU parity of parallax_decode_mla (through the C ABI) against the MLA-style decode oracle
(oracle/mla.py, pinned by tests/test_oracle_mla.py)."""
import numpy as np
import pytest
import torch

from parity import BF16_REL_L2, host, rel_l2

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


@pytest.fixture(scope="module")
def mla():
    from oracle import mla as m

    return m


def _ref(mla, x, seqs=None):
    q, r, c = host(x["q"]), host(x["r"]), host(x["ckv"])
    sl = x["seq_lens"].cpu().numpy() if x.get("seq_lens") is not None else None
    if seqs is not None:
        q, r, c = q[seqs], r[seqs], c[seqs]
        sl = sl[seqs] if sl is not None else None
    return mla.mla_decode(q, r, c, x["d_latent"], x["scale"], sl)


def _check(plx, mla, x, num_splits=0, tol=BF16_REL_L2):
    out = plx.parallax_decode_mla(x["q"], x["r"], x["ckv"], x["scale"], seq_lens=x.get("seq_lens"),
                                  num_splits=num_splits)
    torch.cuda.synchronize()
    got, ref = host(out), _ref(mla, x)
    assert got.shape == ref.shape and np.isfinite(got).all()
    assert rel_l2(got, ref) <= tol, (rel_l2(got, ref), num_splits)
    # per (sequence, head) as well: a wrong column or wave shows up in single rows
    err = np.linalg.norm(got - ref, axis=-1) / np.maximum(np.linalg.norm(ref, axis=-1), 1e-6)
    assert err.max() <= 4 * tol, err.max()
    return got


# Up to 16 columns (heads x rows) take the 16-column kernel, more the 32-column one: the basic
# cases run on both (48 heads: one full group of 32 columns and a half-filled one).
HEADS = [16, 48]


@pytest.mark.parametrize("Hq", HEADS)
@pytest.mark.parametrize("L", [1, 2, 15, 16, 17, 63, 64, 65, 127, 129, 200, 777, 2048])
def test_lengths_and_tails(plx, synth, mla, L, Hq):
    x = synth.mla_decode_inputs(2, Hq, L, seed=4000 + L, device=DEV)
    _check(plx, mla, x, num_splits=1)
    _check(plx, mla, x, num_splits=0)


@pytest.mark.parametrize("Hq", HEADS)
@pytest.mark.parametrize("S", [1, 2, 3, 5, 8, 32, 128])
def test_split_counts_agree_incl_empty_splits(plx, synth, mla, S, Hq):
    x = synth.mla_decode_inputs(2, Hq, 1000, seed=4100, device=DEV)
    got = _check(plx, mla, x, num_splits=S)
    one = host(plx.parallax_decode_mla(x["q"], x["r"], x["ckv"], x["scale"], num_splits=1))
    assert rel_l2(got, one) <= 4e-3       # different summation order, each output rounded to bf16 once


@pytest.mark.parametrize("Hq", [1, 5, 16, 17, 40, 128])
def test_head_counts_and_partial_column_groups(plx, synth, mla, Hq):
    x = synth.mla_decode_inputs(2, Hq, 300, seed=4200 + Hq, device=DEV)
    _check(plx, mla, x)
    _check(plx, mla, x, num_splits=3)


@pytest.mark.parametrize("Hq", HEADS)
def test_ragged_lengths_with_an_empty_sequence(plx, synth, mla, Hq):
    x = synth.mla_decode_inputs(5, Hq, 900, seed=4300, device=DEV, ragged=True)
    x["seq_lens"][2] = 0
    x["seq_lens"][4] = 1
    for S in (0, 1, 4):
        got = _check(plx, mla, x, num_splits=S)
        assert (got[2] == 0).all()
        np.testing.assert_allclose(got[4], np.broadcast_to(host(x["ckv"])[4, 0, :512], got[4].shape), rtol=1e-2, atol=1e-2)


@pytest.mark.parametrize("Hq", HEADS)
def test_strided_cache_and_small_probe(plx, synth, mla, Hq):
    x = synth.mla_decode_inputs(3, Hq, 500, seed=4400, device=DEV, r_scale=0.1)
    wide = torch.zeros(3, 520, 640, dtype=torch.bfloat16, device=DEV)   # rows of 640, 20 spare tokens
    wide[:, :500, :576] = x["ckv"]
    view = wide[:, :500, :576]
    assert not view.is_contiguous()
    a = _check(plx, mla, dict(x, ckv=view))
    b = _check(plx, mla, x)
    np.testing.assert_array_equal(a, b)


@pytest.mark.parametrize("Hq", HEADS)
def test_large_logit_range_and_zero_scale(plx, synth, mla, Hq):
    x = synth.mla_decode_inputs(2, Hq, 700, seed=4500, device=DEV)
    x["q"] = (x["q"].float() * 12.0).to(torch.bfloat16)     # logits spread over ~ +-40: softmax nearly one-hot
    _check(plx, mla, x, num_splits=4)
    _check(plx, mla, dict(x, scale=0.0), num_splits=2)       # uniform weights


@pytest.mark.parametrize("Hq", HEADS)
@pytest.mark.parametrize("rise", [-3000.0, -300.0, 6.0, 40.0, 300.0, 3000.0])
def test_logits_that_drift_along_the_sequence(plx, synth, mla, Hq, rise):
    """Every key carries a component, growing linearly with its position, along a direction all
    queries share: the running maximum of every column rises (or falls) by `rise` (log2 domain)
    over the sequence -- by a fraction of a binade per tile, by a few, by more than ten or by more
    than a hundred, so the softmax reference stays for many tiles, moves now and then, moves in
    every tile, or has to move before the tile's weights can be used at all. The 32-column kernel
    lets its reference lag the maximum by up to eight binades and computes a tile's weights before
    it knows the tile's maximum (up to 64 binades above the reference they stand)."""
    L = 1500
    x = synth.mla_decode_inputs(2, Hq, L, seed=4550 + Hq, device=DEV)
    q = x["q"].float()
    q[..., 0] = 8.0
    x["q"] = q.to(torch.bfloat16)
    x["r"][..., 0] = 0                      # (the probe does not see the drifting component)
    c = x["ckv"].float()
    per_key = rise / (x["scale"] * 8.0 * 1.4426950408889634) / L        # logit = scale * 8 * c[j, 0]
    c[..., 0] = per_key * torch.arange(L, device=DEV, dtype=torch.float32)
    x["ckv"] = c.to(torch.bfloat16)
    for S in (1, 3):
        _check(plx, mla, x, num_splits=S)


@pytest.mark.parametrize("Hq", HEADS)
def test_zero_probe_is_softmax_attention_over_the_latent(plx, synth, mla, Hq):
    x = synth.mla_decode_inputs(2, Hq, 400, seed=4600, device=DEV)
    x["r"] = torch.zeros_like(x["r"])
    got = _check(plx, mla, x)
    q, c = torch.tensor(host(x["q"])), torch.tensor(host(x["ckv"]))
    ref = torch.nn.functional.scaled_dot_product_attention(
        q[:, :, None, :], c[:, None].expand(2, Hq, 400, 576), c[:, None, :, :512].expand(2, Hq, 400, 512),
        scale=x["scale"])[:, :, 0].numpy()
    assert rel_l2(got, ref) <= BF16_REL_L2


def test_deterministic_and_errors(plx, synth):
    x = synth.mla_decode_inputs(2, 16, 1500, seed=4700, device=DEV)
    a = plx.parallax_decode_mla(x["q"], x["r"], x["ckv"], x["scale"])
    b = plx.parallax_decode_mla(x["q"], x["r"], x["ckv"], x["scale"])
    assert torch.equal(a, b)
    with pytest.raises(plx.ParallaxError):                   # only 512 + 64
        plx.parallax_decode_mla(x["q"][..., :320].contiguous(), x["r"][..., :320].contiguous(),
                                x["ckv"][..., :320].contiguous(), x["scale"], d_latent=256)
    with pytest.raises(plx.ParallaxError):
        plx.parallax_decode_mla(x["q"].float(), x["r"].float(), x["ckv"].float(), x["scale"])


def test_serving_shape_sampled(plx, synth, mla):
    """B = 32 sequences of up to 16 384 tokens, 16 heads (one column group, the per-GPU share of a
    128-head model under 8-way head parallelism): all heads of four sampled sequences."""
    x = synth.mla_decode_inputs(32, 16, 16384, seed=4800, device=DEV, ragged=True)
    out = plx.parallax_decode_mla(x["q"], x["r"], x["ckv"], x["scale"], seq_lens=x["seq_lens"])
    torch.cuda.synchronize()
    lens = x["seq_lens"].cpu().numpy()
    seqs = sorted({int(lens.argmin()), int(lens.argmax()), 7, 19})
    ref = _ref(mla, x, seqs)
    assert rel_l2(host(out)[seqs], ref) <= BF16_REL_L2


@pytest.mark.parametrize("case", range(12))
def test_random_shapes(plx, synth, mla, case):
    rng = np.random.default_rng(4900 + case)
    B = int(rng.integers(1, 5))
    Hq = int(rng.choice([1, 3, 8, 16, 24, 33, 64]))
    L = int(rng.choice([1, 31, 64, 100, 255, 256, 257, 600, 1500, 4097]))
    S = int(rng.choice([0, 0, 1, 2, 7, 19]))
    x = synth.mla_decode_inputs(B, Hq, L, seed=4950 + case, device=DEV, ragged=bool(rng.integers(0, 2)),
                                r_scale=float(rng.choice([1.0, 0.2])))
    if rng.integers(0, 2):   # a cache with padded rows and spare tokens
        wide = torch.zeros(B, L + 5, 576 + 64, dtype=torch.bfloat16, device=DEV)
        wide[:, :L, :576] = x["ckv"]
        x["ckv"] = wide[:, :L, :576]
    _check(plx, mla, x, num_splits=S)


@pytest.mark.parametrize("Hq", HEADS)
def test_hip_graph_replays_match_eager(plx, synth, Hq):
    """The two launches of a split step captured once and replayed with new cache contents."""
    import ctypes

    x = synth.mla_decode_inputs(4, Hq, 3000, seed=4990, device=DEV, ragged=True)
    out = torch.empty(4, Hq, 512, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(plx.parallax_decode_mla_workspace_bytes(4, Hq) // 4, dtype=torch.float32, device=DEV)
    a = plx.decode_mla_args(x["q"], x["r"], x["ckv"], out, x["scale"], x["seq_lens"], 6, ws)
    lib = plx.load_library()
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        assert lib.parallax_decode_mla(ctypes.byref(a), int(torch.cuda.current_stream().cuda_stream)) == 0
    torch.cuda.current_stream().wait_stream(side)
    gen = torch.Generator(device=DEV).manual_seed(4991)
    for rep in range(3):
        if rep:
            x["ckv"].copy_(torch.randn(x["ckv"].shape, generator=gen, device=DEV))
            x["q"].copy_(torch.randn(x["q"].shape, generator=gen, device=DEV))
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        eager = plx.parallax_decode_mla(x["q"], x["r"], x["ckv"], x["scale"], seq_lens=x["seq_lens"], num_splits=6)
        torch.cuda.synchronize()
        assert torch.equal(out, eager)


@pytest.mark.parametrize("page_size", [1, 16, 48, 64, 100, 128, 256])
def test_paged_cache_matches_contiguous(plx, synth, mla, page_size):
    """The same tokens behind a block table (random page order, spare pages, a ragged batch):
    the same bits as the contiguous cache, for page sizes fetched page-wise (multiples of 64)
    and row by row (the others)."""
    x = synth.mla_decode_inputs(3, 20, 700, seed=5000 + page_size, device=DEV, ragged=True)
    x["seq_lens"][1] = 700
    want = _check(plx, mla, x, num_splits=3)
    pool, table = synth.mla_paged_cache(x, page_size, seed=5001)
    for S in (3, 1):
        got = plx.parallax_decode_mla(x["q"], x["r"], pool, x["scale"], seq_lens=x["seq_lens"], num_splits=S,
                                      block_table=table, max_len=700)
        torch.cuda.synchronize()
        if S == 3:
            np.testing.assert_array_equal(host(got), want)
        else:
            assert rel_l2(host(got), _ref(mla, x)) <= BF16_REL_L2
    # a pool with padded rows and a wider table than needed
    wide = torch.zeros(pool.shape[0], page_size, 640, dtype=torch.bfloat16, device=DEV)
    wide[..., :576] = pool
    table2 = torch.cat([table, torch.full_like(table[:, :2], 10 ** 6)], dim=1).contiguous()   # out-of-range entries: clamped, never read
    got = plx.parallax_decode_mla(x["q"], x["r"], wide[..., :576], x["scale"], seq_lens=x["seq_lens"], num_splits=3,
                                  block_table=table2, max_len=700)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(got), want)


# ---- several query rows per head, sliding window, prefill over the latent cache ----------------
def _rows_inputs(synth, B, Hq, Tq, L, seed, ragged=False):
    x = synth.mla_decode_inputs(B, Hq * Tq, L, seed=seed, device=DEV, ragged=ragged)
    x["q"] = x["q"].view(B, Hq, Tq, -1)
    x["r"] = x["r"].view(B, Hq, Tq, -1)
    return x


def _check_rows(plx, mla, x, window=0, num_splits=0, paged=None, tol=BF16_REL_L2):
    kw = {}
    ckv = x["ckv"]
    if paged is not None:
        ckv, kw["block_table"], kw["max_len"] = paged[0], paged[1], x["ckv"].shape[1]
    out = plx.parallax_decode_mla(x["q"], x["r"], ckv, x["scale"], seq_lens=x.get("seq_lens"),
                                  num_splits=num_splits, window=window, **kw)
    torch.cuda.synchronize()
    sl = x["seq_lens"].cpu().numpy() if x.get("seq_lens") is not None else None
    ref = mla.mla_rows(host(x["q"]), host(x["r"]), host(x["ckv"]), x["d_latent"], x["scale"], sl, window=window)
    got = host(out)
    assert got.shape == ref.shape and np.isfinite(got).all()
    assert rel_l2(got, ref) <= tol, (rel_l2(got, ref), window, num_splits)
    norm = np.linalg.norm(ref, axis=-1)
    err = np.linalg.norm(got - ref, axis=-1)[norm > 0] / norm[norm > 0]
    assert err.max() <= 4 * tol, err.max()
    assert (got[norm == 0] == 0).all()        # rows that see no token: zeros, exactly
    return got


@pytest.mark.parametrize("Hq,Tq,L", [(16, 2, 300), (16, 4, 1000), (5, 3, 129), (2, 8, 64), (1, 16, 500),
                                      (3, 7, 70), (16, 5, 4)])
def test_several_query_rows_at_the_last_positions(plx, synth, mla, Hq, Tq, L):
    """Row t of a head sees the tokens up to position L - Tq + t: every (head, row) pair is a
    column of its own; L < Tq leaves the first rows without a token."""
    x = _rows_inputs(synth, 2, Hq, Tq, L, seed=4600 + L)
    _check_rows(plx, mla, x, num_splits=1)
    _check_rows(plx, mla, x, num_splits=0)
    _check_rows(plx, mla, x, num_splits=3)


def test_several_query_rows_ragged_and_paged(plx, synth, mla):
    x = _rows_inputs(synth, 5, 8, 4, 900, seed=4700, ragged=True)
    x["seq_lens"][1] = 0
    x["seq_lens"][2] = 2                       # shorter than Tq
    _check_rows(plx, mla, x)
    _check_rows(plx, mla, x, num_splits=4)
    pool, table = synth.mla_paged_cache(x, 64, seed=4701)
    _check_rows(plx, mla, x, paged=(pool, table))
    pool, table = synth.mla_paged_cache(x, 48, seed=4702)
    _check_rows(plx, mla, x, window=100, paged=(pool, table))


@pytest.mark.parametrize("Tq,L,W", [(1, 1000, 1), (1, 1000, 64), (1, 1000, 65), (1, 1000, 300), (1, 300, 5000),
                                     (4, 1000, 130), (3, 200, 2), (8, 2048, 1000)])
def test_sliding_window(plx, synth, mla, Tq, L, W):
    """A row sees its own position and the W - 1 before it: the tiles before the earliest window
    of the workgroup's columns are not visited."""
    x = _rows_inputs(synth, 2, 16, Tq, L, seed=4800 + L + W)
    _check_rows(plx, mla, x, window=W, num_splits=1)
    _check_rows(plx, mla, x, window=W, num_splits=0)
    _check_rows(plx, mla, x, window=W, num_splits=5)


@pytest.mark.parametrize("Hq,Tq,L,W", [(48, 1, 1000, 1), (48, 1, 1000, 65), (48, 1, 1000, 300), (40, 2, 700, 130),
                                        (17, 1, 300, 5000)])
def test_sliding_window_with_more_than_16_columns(plx, synth, mla, Hq, Tq, L, W):
    """The same on the 32-column kernel with one row per head (above, only several rows per head
    reach it): full and half-filled column groups, ragged lengths."""
    x = _rows_inputs(synth, 3, Hq, Tq, L, seed=4850 + L + W, ragged=True)
    for S in (1, 0, 3):
        _check_rows(plx, mla, x, window=W, num_splits=S)


@pytest.mark.parametrize("Hq,T,W", [(2, 300, 0), (4, 513, 0), (1, 1000, 0), (3, 400, 100)])
def test_causal_prefill_over_the_latent_cache(plx, synth, mla, Hq, T, W):
    """Tq = the prompt length: every row of the prompt attends to the latent rows up to its own."""
    x = _rows_inputs(synth, 2, Hq, T, T, seed=4900 + T)
    _check_rows(plx, mla, x, window=W)
    # a chunk of 128 rows behind 500 cached tokens
    x = _rows_inputs(synth, 1, Hq, 128, 628, seed=4901 + T)
    _check_rows(plx, mla, x, window=W)


def test_rows_and_window_arguments_are_validated(plx, synth):
    import ctypes

    x = _rows_inputs(synth, 1, 4, 2, 100, seed=4950)
    out = torch.empty(1, 4, 2, 512, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(8 * 4 * 1028, dtype=torch.float32, device=DEV)
    lib, sptr = plx.load_library(), int(torch.cuda.current_stream().cuda_stream)
    a = plx.decode_mla_args(x["q"], x["r"], x["ckv"], out, x["scale"], None, 4, ws)
    assert lib.parallax_decode_mla(ctypes.byref(a), sptr) == 0
    a.window = -1
    assert lib.parallax_decode_mla(ctypes.byref(a), sptr) == plx.PLX_ERR_SHAPE
    a.window, a.Tq = 0, -2
    assert lib.parallax_decode_mla(ctypes.byref(a), sptr) == plx.PLX_ERR_SHAPE
    a.Tq, a.num_splits = 2, 8                  # the workspace holds 4 splits of 8 columns
    assert lib.parallax_decode_mla(ctypes.byref(a), sptr) == plx.PLX_ERR_WORKSPACE
    torch.cuda.synchronize()


def test_many_heads_and_rows_at_the_benchmark_launches(plx, synth, mla):
    """The launches bench.py times: B=16 x 128 heads x L=8192 (four groups of 32 columns per sequence,
    heuristic splits), 4 rows x 16 heads at the end of L=16384, and the causal prefill of 4096
    latent rows -- the oracle on sampled sequences / rows."""
    x = synth.mla_decode_inputs(16, 128, 8192, seed=4960, device=DEV)
    out = plx.parallax_decode_mla(x["q"], x["r"], x["ckv"], x["scale"])
    torch.cuda.synchronize()
    seqs = [0, 7, 15]
    assert rel_l2(host(out)[seqs], _ref(mla, x, seqs)) <= BF16_REL_L2

    x = _rows_inputs(synth, 8, 16, 4, 16384, seed=4961)
    out = plx.parallax_decode_mla(x["q"], x["r"], x["ckv"], x["scale"])
    torch.cuda.synchronize()
    for b in (0, 5):
        ref = mla.mla_rows(host(x["q"][b:b + 1]), host(x["r"][b:b + 1]), host(x["ckv"][b:b + 1]), 512, x["scale"])
        assert rel_l2(host(out[b:b + 1]), ref) <= BF16_REL_L2

    T = 4096
    x = _rows_inputs(synth, 1, 16, T, T, seed=4962)
    out = host(plx.parallax_decode_mla(x["q"], x["r"], x["ckv"], x["scale"]))
    assert np.isfinite(out).all()
    rng = np.random.default_rng(4963)
    # a row of every 16-row workgroup of two heads, the first and last 32 rows of another
    picks = [(h, int(rng.integers(blk, blk + 16))) for h in (0, 9) for blk in range(0, T, 16)]
    picks += [(15, t) for t in list(range(32)) + list(range(T - 32, T))]
    c = host(x["ckv"])
    q, r = host(x["q"]), host(x["r"])
    err2 = ref2 = 0.0
    for (h, t) in picks:
        one = mla.mla_decode(q[:, h:h + 1, t], r[:, h:h + 1, t], c, 512, x["scale"], np.array([t + 1]))[0, 0]
        err2 += float(((out[0, h, t] - one) ** 2).sum())
        ref2 += float((one ** 2).sum())
        assert np.linalg.norm(out[0, h, t] - one) <= 4e-2 * np.linalg.norm(one), (h, t)
    assert (err2 / ref2) ** 0.5 <= BF16_REL_L2
