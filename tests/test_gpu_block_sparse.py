"""GPU parity of block-sparse parallax_prefill and parallax_prefill_backward (through the C ABI)
against the arbitrary-mask oracle: each 128-row block visits a listed subset of the 64-key tiles."""
import numpy as np
import pytest
import torch

from parity import BF16_REL_L2, assert_gradient_close, host, rel_l2

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
def masked():
    from oracle import masked as m

    return m


def _ref(masked, y, bm, causal):
    q, r, k, v = (host(y[n]) for n in "qrkv")
    dense = masked.block_mask_to_dense(bm, q.shape[2], k.shape[2], 128, 64, causal)
    return masked.masked_forward(q, r, k, v, y["scale"], dense), dense


def _check(plx, masked, y, bm, causal):
    out = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=causal,
                               block_mask=torch.as_tensor(bm, device=DEV))
    torch.cuda.synchronize()
    got = host(out)
    ref, dense = _ref(masked, y, bm, causal)
    assert np.isfinite(got).all()
    assert rel_l2(got, ref) <= BF16_REL_L2
    empty = ~np.broadcast_to(dense, got.shape[:3] + dense.shape[-1:]).any(axis=-1)
    assert (got[empty] == 0).all()          # rows that see nothing are zeros, exactly
    live = ~empty
    row_err = np.linalg.norm(got - ref, axis=-1)[live] / np.maximum(np.linalg.norm(ref, axis=-1)[live], 1e-6)
    assert row_err.max() <= 8 * BF16_REL_L2
    return got


@pytest.mark.parametrize("T,Tkv", [(128, 128), (300, 300), (1000, 1000), (200, 900), (640, 2048)])
@pytest.mark.parametrize("causal", [True, False])
def test_random_block_masks_shared_by_all_heads(plx, synth, masked, T, Tkv, causal):
    y = synth.prefill_inputs(2, 4, 2, Tkv, 128, seed=3000 + T, device=DEV)
    if Tkv > T:
        y["q"], y["r"] = y["q"][:, :, Tkv - T:].contiguous(), y["r"][:, :, Tkv - T:].contiguous()
    rng = np.random.default_rng(3001 + T)
    nrb, nkt = -(-T // 128), -(-Tkv // 64)
    bm = rng.random((nrb, nkt)) < 0.35
    bm[0, :] |= np.arange(nkt) == 0          # keep row block 0 alive in the causal case
    _check(plx, masked, y, bm, causal)


@pytest.mark.parametrize("causal,density", [(True, 0.85), (False, 0.85), (True, 0.2)])
def test_long_rows_take_the_unmasked_tile_loop(plx, synth, masked, causal, density):
    """Many listed tiles are visible to a whole row block: those go through the branch-free
    pipeline, the diagonal and the ragged last tile through the masked one. One batch entry of
    benchmark configuration 4 (T = 4096, d = 128), two KV heads' groups."""
    y = synth.prefill_inputs(1, 4, 2, 4096 - 37, 128, seed=3500, device=DEV)
    rng = np.random.default_rng(3501)
    bm = rng.random((32, 64)) < density
    bm[:, 0] = True
    _check(plx, masked, y, bm, causal)


def test_per_batch_and_per_head_masks_with_empty_row_blocks(plx, synth, masked):
    B, Hq, T = 2, 4, 700
    y = synth.prefill_inputs(B, Hq, 2, T, 128, seed=3100, device=DEV)
    rng = np.random.default_rng(3101)
    nrb, nkt = -(-T // 128), -(-T // 64)
    bm = rng.random((B, Hq, nrb, nkt)) < 0.3
    bm[0, 1, 2] = False                       # an empty row block
    bm[1, 3] = False                          # a head that sees nothing at all
    _check(plx, masked, y, bm, True)
    # per head only (shared by the batch), full attention, d = 64
    y = synth.prefill_inputs(B, Hq, 4, 500, 64, seed=3102, device=DEV)
    bm = rng.random((1, Hq, 4, 8)) < 0.5
    _check(plx, masked, y, bm, False)


def test_all_tiles_listed_is_dense_attention_and_a_band_is_a_window(plx, synth, masked, oracle):
    y = synth.prefill_inputs(1, 4, 2, 900, 128, seed=3200, device=DEV)
    nrb, nkt = 8, 15
    got = _check(plx, masked, y, np.ones((nrb, nkt), bool), True)
    dense = host(plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=True))
    assert rel_l2(got, dense) <= 2e-3         # same keys, different row-sum rounding path
    # block band: row block i sees its own two tiles and the four before (a blocky window)
    bm = np.zeros((nrb, nkt), bool)
    for i in range(nrb):
        bm[i, max(0, 2 * i - 4): 2 * i + 2] = True
    _check(plx, masked, y, bm, True)


def test_wide_logit_range_takes_the_safe_path(plx, synth, masked):
    """The fixed softmax reference comes from the first listed block, which some rows do not see:
    with scores spread over hundreds of binary orders of magnitude it overflows or underflows
    and the kernel must fall back to the online-rescale pass."""
    y = synth.prefill_inputs(1, 4, 2, 700, 128, seed=3300, device=DEV)
    y["q"] = (y["q"].float() * 20.0).to(torch.bfloat16)
    ramp = torch.linspace(3.0, 0.2, 700, device=DEV).view(1, 1, 700, 1)
    y["k"] = (y["k"].float() * ramp).to(torch.bfloat16)
    rng = np.random.default_rng(3301)
    bm = rng.random((6, 11)) < 0.5
    bm[:, 0] = True
    out = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=True,
                               block_mask=torch.as_tensor(bm, device=DEV))
    torch.cuda.synchronize()
    ref, _ = _ref(masked, y, bm, True)
    assert np.isfinite(host(out)).all() and rel_l2(host(out), ref) <= BF16_REL_L2


LOG2E = 1.4426950408889634


def _check_backward(plx, synth, masked, y, bm, causal, seed):
    """Forward with the row cache, then the gradients, under the block mask: cache and gradients
    against the arbitrary-mask oracle (closed forms of App. D over the allowed pairs)."""
    B, Hq, T, d = y["q"].shape
    g = synth.prefill_inputs(B, Hq, k_heads(y), T, d, seed=seed, device=DEV)["q"].contiguous()
    mask_t = torch.as_tensor(bm, device=DEV)
    o, vbar, stats = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=causal,
                                          block_mask=mask_t, save_for_backward=True)
    grads = plx.parallax_prefill_backward(y["q"], y["r"], y["k"], y["v"], o, vbar, stats, g, y["scale"],
                                          causal=causal, block_mask=mask_t)
    torch.cuda.synchronize()
    hq, hr, hk, hv = (host(y[n]) for n in "qrkv")
    dense = masked.block_mask_to_dense(bm, T, hk.shape[2], 128, 64, causal)
    ro, rvbar, rubar, rlog = masked.masked_forward_with_cache(hq, hr, hk, hv, y["scale"], dense)
    live = np.broadcast_to(dense, (B, Hq) + dense.shape[-2:]).any(axis=-1)
    assert rel_l2(host(o), ro) <= BF16_REL_L2 and rel_l2(host(vbar), rvbar) <= BF16_REL_L2
    st = host(stats)
    np.testing.assert_allclose(st[..., 0][live], (rlog * LOG2E)[live], rtol=0, atol=2e-2)
    assert np.abs(st[..., 1][live] - rubar[live]).max() <= 2e-2 * max(1.0, np.abs(rubar).max())
    assert np.isposinf(st[..., 0][~live]).all() and (st[..., 1][~live] == 0).all()
    assert (host(vbar)[~live] == 0).all() and (host(o)[~live] == 0).all()
    want = masked.masked_backward(hq, hr, hk, hv, host(g), y["scale"], dense)
    for name, got, ref in zip(("dq", "dr", "dk", "dv"), grads, want):
        assert_gradient_close(name, host(got), ref, BF16_REL_L2, (tuple(y["q"].shape), causal))
    # rows and keys outside every listed cell: zero gradients, exactly
    assert (host(grads[0])[~live] == 0).all() and (host(grads[1])[~live] == 0).all()
    G = Hq // hk.shape[1]
    seen = np.broadcast_to(dense, (B, Hq) + dense.shape[-2:]).any(axis=-2).reshape(B, -1, G, hk.shape[2]).any(axis=2)
    assert (host(grads[2])[~seen] == 0).all() and (host(grads[3])[~seen] == 0).all()
    return grads


def k_heads(y):
    return y["k"].shape[1]


@pytest.mark.parametrize("T,Tkv", [(128, 128), (300, 300), (1000, 1000), (200, 900), (640, 2048)])
@pytest.mark.parametrize("causal", [True, False])
def test_backward_random_block_masks_shared_by_all_heads(plx, synth, masked, T, Tkv, causal):
    y = synth.prefill_inputs(2, 4, 2, Tkv, 128, seed=3000 + T, device=DEV)
    if Tkv > T:
        y["q"], y["r"] = y["q"][:, :, Tkv - T:].contiguous(), y["r"][:, :, Tkv - T:].contiguous()
    rng = np.random.default_rng(3001 + T)
    nrb, nkt = -(-T // 128), -(-Tkv // 64)
    bm = rng.random((nrb, nkt)) < 0.35
    bm[0, :] |= np.arange(nkt) == 0
    _check_backward(plx, synth, masked, y, bm, causal, seed=3600 + T)


def test_backward_per_batch_and_per_head_masks_with_empty_blocks(plx, synth, masked):
    B, Hq, T = 2, 4, 700
    y = synth.prefill_inputs(B, Hq, 2, T, 128, seed=3100, device=DEV)
    rng = np.random.default_rng(3101)
    nrb, nkt = -(-T // 128), -(-T // 64)
    bm = rng.random((B, Hq, nrb, nkt)) < 0.3
    bm[0, 1, 2] = False                       # an empty row block
    bm[1, 3] = False                          # a head that sees nothing at all
    bm[:, :, :, 4:6] = False                  # a key block nobody lists
    _check_backward(plx, synth, masked, y, bm, True, seed=3610)
    # per head only (shared by the batch), full attention, d = 64, one KV head per query head
    y = synth.prefill_inputs(B, Hq, 4, 500, 64, seed=3102, device=DEV)
    bm = rng.random((1, Hq, 4, 8)) < 0.5
    _check_backward(plx, synth, masked, y, bm, False, seed=3611)
    # a group of four query heads with their own masks over one KV head, odd number of key tiles
    y = synth.prefill_inputs(1, 4, 1, 450, 64, seed=3103, device=DEV)
    bm = rng.random((1, 4, 4, 8)) < 0.4
    _check_backward(plx, synth, masked, y, bm, True, seed=3612)


def test_backward_all_tiles_listed_is_the_dense_backward_and_a_block_band(plx, synth, masked):
    y = synth.prefill_inputs(1, 4, 2, 900, 128, seed=3200, device=DEV)
    nrb, nkt = 8, 15
    grads = _check_backward(plx, synth, masked, y, np.ones((nrb, nkt), bool), True, seed=3620)
    g = synth.prefill_inputs(1, 4, 2, 900, 128, seed=3620, device=DEV)["q"].contiguous()
    o, vbar, stats = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=True,
                                          save_for_backward=True)
    dense = plx.parallax_prefill_backward(y["q"], y["r"], y["k"], y["v"], o, vbar, stats, g, y["scale"], causal=True)
    torch.cuda.synchronize()
    for a, b in zip(grads, dense):
        assert rel_l2(host(a), host(b).astype(np.float64)) <= 4e-3   # same pairs, other tile order
    bm = np.zeros((nrb, nkt), bool)
    for i in range(nrb):
        bm[i, max(0, 2 * i - 4): 2 * i + 2] = True
    _check_backward(plx, synth, masked, y, bm, True, seed=3621)


def test_backward_block_lists_are_validated(plx, synth):
    y = synth.prefill_inputs(1, 4, 2, 256, 128, seed=3400, device=DEV)
    o, vbar, stats = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], save_for_backward=True)
    with pytest.raises(ValueError):
        plx.parallax_prefill_backward(y["q"], y["r"], y["k"], y["v"], o, vbar, stats, o, y["scale"],
                                      block_mask=torch.ones(3, 4, device=DEV))
    with pytest.raises(plx.ParallaxError):    # no window together with block lists
        plx.parallax_prefill_backward(y["q"], y["r"], y["k"], y["v"], o, vbar, stats, o, y["scale"], window=64,
                                      block_mask=torch.ones(2, 4, device=DEV))
    # some of the four arrays missing
    import ctypes
    ws = torch.empty(4 * 256 * 4, dtype=torch.float32, device=DEV)
    dq, dk = torch.empty_like(o), torch.empty_like(y["k"])
    a = plx.prefill_bwd_args(y["q"], y["r"], y["k"], y["v"], o, vbar, stats, o, dq, dq.clone(), dk, dk.clone(),
                             y["scale"], True, ws)
    row_ptr, tile_idx, Bs, Hs = plx.block_mask_lists(torch.ones(2, 4, device=DEV))
    a.sparse_row_ptr, a.sparse_tile_idx, a.sparse_batch, a.sparse_heads = row_ptr.data_ptr(), tile_idx.data_ptr(), Bs, Hs
    st = plx.load_library().parallax_prefill_backward(ctypes.byref(a), int(torch.cuda.current_stream().cuda_stream))
    assert st == plx.PLX_ERR_NULL


def test_sparse_lists_are_validated(plx, synth):
    y = synth.prefill_inputs(1, 4, 2, 256, 128, seed=3400, device=DEV)
    with pytest.raises(ValueError):
        plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], block_mask=torch.ones(3, 4, device=DEV))
    with pytest.raises(plx.ParallaxError):    # no window together with a block mask
        plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], window=64,
                             block_mask=torch.ones(2, 4, device=DEV))


def test_backward_at_the_benchmark_launch(plx, synth, masked):
    """The block-sparse backward bench.py times (config-4 shape, causal, a random quarter of the
    tiles): the gradients of two (batch, KV head) pairs of that launch against the oracle."""
    B, Hq, Hkv, T, d = 4, 16, 8, 4096, 128
    y = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=1010, device=DEV)
    g = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=3700, device=DEV)["q"].contiguous()
    nrb, nkt = T // 128, T // 64
    bm = np.random.default_rng(1011).random((nrb, nkt)) < 0.25
    bm &= np.arange(nkt)[None, :] <= 2 * np.arange(nrb)[:, None] + 1
    bm[5] = False                                   # a row block that lists nothing
    mask_t = torch.as_tensor(bm, device=DEV)
    o, vbar, stats = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=True,
                                          block_mask=mask_t, save_for_backward=True)
    grads = plx.parallax_prefill_backward(y["q"], y["r"], y["k"], y["v"], o, vbar, stats, g, y["scale"],
                                          causal=True, block_mask=mask_t)
    torch.cuda.synchronize()
    dense = masked.block_mask_to_dense(bm, T, T, 128, 64, True)
    for b, hk in ((0, 3), (3, 6)):
        qs, ks = slice(2 * hk, 2 * hk + 2), slice(hk, hk + 1)
        want = masked.masked_backward(host(y["q"][b:b + 1, qs]), host(y["r"][b:b + 1, qs]),
                                      host(y["k"][b:b + 1, ks]), host(y["v"][b:b + 1, ks]), host(g[b:b + 1, qs]),
                                      y["scale"], dense)
        for name, got, ref, hs in zip(("dq", "dr", "dk", "dv"), grads, want, (qs, qs, ks, ks)):
            assert_gradient_close(name, host(got[b:b + 1, hs]), ref, BF16_REL_L2, (b, hk))
