"""GPU parity of parallax_prefill_backward (through the C ABI) against the backward oracle
(closed forms of the paper's App. D in float64, pinned by tests/test_oracle_backward.py), and of
the row cache the forward writes for it."""
import numpy as np
import pytest
import torch

from parity import BF16_REL_L2, F32_MAX_REL, assert_gradient_close, host, max_rel, rel_l2

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
LOG2E = 1.4426950408889634


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
def bwd_oracle():
    from oracle import parallax_backward

    return parallax_backward


def _inputs(synth, B, Hq, Hkv, T, Tkv, d, seed, r_scale=1.0):
    y = synth.prefill_inputs(B, Hq, Hkv, Tkv, d, seed=seed, device=DEV, r_scale=r_scale)
    if Tkv > T:
        y["q"], y["r"] = y["q"][:, :, Tkv - T:].contiguous(), y["r"][:, :, Tkv - T:].contiguous()
    g = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=seed + 1, device=DEV)["q"].contiguous()  # N(0,1) bf16
    return y, g


def _run(plx, y, g, causal, window=0):
    o, vbar, stats = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=causal,
                                          save_for_backward=True, window=window)
    grads = plx.parallax_prefill_backward(y["q"], y["r"], y["k"], y["v"], o, vbar, stats, g, y["scale"],
                                          causal=causal, window=window)
    torch.cuda.synchronize()
    return o, vbar, stats, grads


def _check(plx, synth, bwd_oracle, B, Hq, Hkv, T, Tkv, d, causal, seed, r_scale=1.0, tol=BF16_REL_L2, window=0):
    y, g = _inputs(synth, B, Hq, Hkv, T, Tkv, d, seed, r_scale)
    _, _, _, grads = _run(plx, y, g, causal, window)
    want = bwd_oracle.backward(*(host(y[n]) for n in "qrkv"), host(g), y["scale"], causal=causal, window=window)
    for name, got, ref in zip(("dq", "dr", "dk", "dv"), grads, want):
        assert_gradient_close(name, host(got), ref, tol, (B, Hq, Hkv, T, Tkv, d, causal, window))


@pytest.mark.parametrize("T", [1, 2, 3, 5, 31, 64, 65, 128, 129, 300, 513])
@pytest.mark.parametrize("causal", [True, False])
def test_backward_small_lengths(plx, synth, bwd_oracle, T, causal):
    # One key per row: the weight 1 + ubar - u is 1, dQ = dR = 0. The forward's row cache holds
    # ubar from the unrounded fp32 P2, so nothing but fp32 rounding is left of ubar - u.
    _check(plx, synth, bwd_oracle, 2, 4, 2, T, T, 128, causal, seed=2000 + T)


@pytest.mark.parametrize("Hq,Hkv,d", [(2, 2, 128), (8, 2, 128), (8, 1, 128), (6, 2, 64), (4, 4, 64), (16, 1, 128), (12, 1, 64)])
def test_backward_gqa_groups_and_head_dims(plx, synth, bwd_oracle, Hq, Hkv, d):
    """The gradients of a KV head add up over the query heads of its group."""
    _check(plx, synth, bwd_oracle, 2, Hq, Hkv, 200, 200, d, True, seed=2100 + Hq + d)


@pytest.mark.parametrize("T,Tkv,causal", [(128, 1000, True), (200, 777, True), (5, 300, True), (100, 333, False)])
def test_backward_more_keys_than_rows(plx, synth, bwd_oracle, T, Tkv, causal):
    _check(plx, synth, bwd_oracle, 1, 8, 2, T, Tkv, 128, causal, seed=2200 + T)


@pytest.mark.parametrize("T,Tkv,W,d", [(300, 300, 1, 128), (300, 300, 2, 128), (300, 300, 3, 64), (300, 300, 7, 128),
                                        (300, 300, 16, 64), (300, 300, 64, 128),
                                        (513, 513, 100, 128), (513, 513, 128, 128), (513, 513, 200, 64),
                                        (1000, 1000, 333, 128), (200, 777, 150, 128), (640, 2048, 512, 128),
                                        (130, 1500, 40, 64), (300, 300, 5000, 128)])
def test_backward_sliding_window(plx, synth, bwd_oracle, T, Tkv, W, d):
    """Rows see their own position and the W - 1 before it: key tiles before the window are
    skipped in the row pass, row tiles after it in the column pass (key blocks nobody sees get
    zero gradients), the edges take the masked pipeline."""
    _check(plx, synth, bwd_oracle, 2, 4, 2, T, Tkv, d, True, seed=2900 + T + W, window=W)


def test_backward_sliding_window_fp32_and_row_cache(plx, synth, bwd_oracle):
    for (T, Tkv, W, d) in [(130, 130, 33, 64), (77, 300, 50, 32)]:
        y = synth.prefill_inputs(2, 4, 2, Tkv, d, seed=2950 + T, dtype=torch.float32, device=DEV)
        if Tkv > T:
            y["q"], y["r"] = y["q"][:, :, Tkv - T:].contiguous(), y["r"][:, :, Tkv - T:].contiguous()
        g = synth.prefill_inputs(2, 4, 2, T, d, seed=2951, dtype=torch.float32, device=DEV)["q"].contiguous()
        _, vbar, stats, grads = _run(plx, y, g, True, W)
        hq, hr, hk, hv = (host(y[n]) for n in "qrkv")
        _, vb, ub, lw = bwd_oracle.forward_with_cache(hq, hr, hk, hv, y["scale"], causal=True, window=W)
        assert max_rel(host(vbar), vb) <= F32_MAX_REL
        np.testing.assert_allclose(host(stats)[..., 0], lw * LOG2E, rtol=0, atol=1e-4)
        want = bwd_oracle.backward(hq, hr, hk, hv, host(g), y["scale"], causal=True, window=W)
        for name, got, ref in zip(("dq", "dr", "dk", "dv"), grads, want):
            assert np.abs(host(got) - ref).max() <= F32_MAX_REL * max(np.abs(ref).max(), 1.0), name
    # bf16 row cache under a window
    y, g = _inputs(synth, 2, 4, 2, 400, 400, 128, 2960)
    o, vbar, stats, _ = _run(plx, y, g, True, 100)
    plain = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=True, window=100)
    np.testing.assert_array_equal(host(o), host(plain))
    _, vb, ub, lw = bwd_oracle.forward_with_cache(*(host(y[n]) for n in "qrkv"), y["scale"], causal=True, window=100)
    assert rel_l2(host(vbar), vb) <= BF16_REL_L2
    np.testing.assert_allclose(host(stats)[..., 0], lw * LOG2E, rtol=0, atol=2e-2)
    assert rel_l2(host(stats)[..., 1], ub) <= BF16_REL_L2


@pytest.mark.parametrize("T,Tkv,causal,window,d", [(300, 300, True, 0, 128), (200, 500, True, 64, 128),
                                                    (257, 257, False, 0, 64), (1100, 1100, True, 0, 128)])
def test_backward_strided_views_equal_dense_tensors(plx, synth, T, Tkv, causal, window, d):
    """q, rho, k, v as views of fused projections laid out [B, T, heads * d], d_o / o / vbar and
    the gradients in [B, T, H, d] order: same bits as the dense [B, H, T, d] call."""
    B, Hq, Hkv = 2, 4, 2
    y, g = _inputs(synth, B, Hq, Hkv, T, Tkv, d, 2990 + T)
    o, vbar, stats = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=causal,
                                          save_for_backward=True, window=window)
    dense = plx.parallax_prefill_backward(y["q"], y["r"], y["k"], y["v"], o, vbar, stats, g, y["scale"],
                                          causal=causal, window=window)

    def bthd(x):                      # same values, [B, T, H, d] in memory, viewed as [B, H, T, d]
        return x.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)

    qr = torch.cat([y["q"].permute(0, 2, 1, 3), y["r"].permute(0, 2, 1, 3)], dim=2).contiguous()   # [B, T, 2 Hq, d]
    kv = torch.cat([y["k"].permute(0, 2, 1, 3), y["v"].permute(0, 2, 1, 3)], dim=2).contiguous()   # [B, Tkv, 2 Hkv, d]
    q2, r2 = qr[:, :, :Hq].permute(0, 2, 1, 3), qr[:, :, Hq:].permute(0, 2, 1, 3)
    k2, v2 = kv[:, :, :Hkv].permute(0, 2, 1, 3), kv[:, :, Hkv:].permute(0, 2, 1, 3)
    assert not q2.is_contiguous() and q2.stride(2) == 2 * Hq * d
    dqr = torch.zeros_like(qr)
    dkv = torch.zeros_like(kv)
    outs = (dqr[:, :, :Hq].permute(0, 2, 1, 3), dqr[:, :, Hq:].permute(0, 2, 1, 3),
            dkv[:, :, :Hkv].permute(0, 2, 1, 3), dkv[:, :, Hkv:].permute(0, 2, 1, 3))
    ws = torch.empty(plx.parallax_prefill_backward_workspace_bytes(B, Hq, T) // 4, dtype=torch.float32, device=DEV)
    a = plx.prefill_bwd_args(q2, r2, k2, v2, bthd(o), bthd(vbar), stats, bthd(g), *outs, y["scale"], causal, ws,
                             window)
    st = plx.load_library().parallax_prefill_backward(__import__("ctypes").byref(a),
                                                      int(torch.cuda.current_stream().cuda_stream))
    assert st == 0
    torch.cuda.synchronize()
    for name, got, ref in zip(("dq", "dr", "dk", "dv"), outs, dense):
        assert torch.equal(got.contiguous(), ref), name


def test_backward_small_probe_and_zero_probe(plx, synth, bwd_oracle):
    _check(plx, synth, bwd_oracle, 1, 4, 2, 400, 400, 128, True, seed=2300, r_scale=0.1)
    # R = 0: dQ, dK, dV are those of softmax attention; dR is the value/key covariance term
    y, g = _inputs(synth, 1, 4, 2, 300, 300, 128, 2301)
    y["r"] = torch.zeros_like(y["r"])
    _, _, _, grads = _run(plx, y, g, True)
    want = bwd_oracle.backward(*(host(y[n]) for n in "qrkv"), host(g), y["scale"], causal=True)
    for got, ref in zip(grads, want):
        assert rel_l2(host(got), ref) <= BF16_REL_L2


def test_forward_row_cache(plx, synth, bwd_oracle):
    """save_for_backward changes nothing in o and adds vbar = sum_j p_j v_j, the log-sum-exp of
    the scaled scores (exp2 domain) and ubar."""
    for causal in (True, False):
        y, g = _inputs(synth, 2, 4, 2, 333, 333, 128, 2400)
        o, vbar, stats, _ = _run(plx, y, g, causal)
        plain = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=causal)
        np.testing.assert_array_equal(host(o), host(plain))
        _, vb, ub, lw = bwd_oracle.forward_with_cache(*(host(y[n]) for n in "qrkv"), y["scale"], causal=causal)
        assert rel_l2(host(vbar), vb) <= BF16_REL_L2
        st = host(stats)
        np.testing.assert_allclose(st[..., 0], lw * LOG2E, rtol=0, atol=2e-2)
        assert rel_l2(st[..., 1], ub) <= BF16_REL_L2


def test_backward_is_deterministic_and_conserves(plx, synth):
    y, g = _inputs(synth, 2, 8, 2, 500, 500, 128, 2500)
    _, _, _, a = _run(plx, y, g, True)
    _, _, _, b = _run(plx, y, g, True)
    for x, z in zip(a, b):
        assert torch.equal(x, z)
    # key-translation invariance of the forward: sum_j dK_j = 0 (up to bf16 rounding of 500 terms);
    # value translation: sum_j dV_j = sum_i dO_i per KV head
    dk, dv = a[2].float(), a[3].float()
    assert dk.sum(dim=2).abs().max().item() <= 2e-2 * dk.abs().sum(dim=2).max().item()
    want = g.float().reshape(2, 2, 4, 500, 128).sum(dim=(2, 3))
    assert (dv.sum(dim=2) - want).abs().max().item() <= 2e-2 * want.abs().max().item() + 0.5


def test_backward_config4_shape_sampled(plx, synth, bwd_oracle):
    """One batch entry of benchmark configuration 4 (T = 4096, 16 query / 8 KV heads, d = 128): full
    oracle gradients of two KV heads' groups against the kernel's."""
    y, g = _inputs(synth, 1, 4, 2, 4096, 4096, 128, 2600)
    _, _, _, grads = _run(plx, y, g, True)
    want = bwd_oracle.backward(*(host(y[n]) for n in "qrkv"), host(g), y["scale"], causal=True)
    for name, got, ref in zip(("dq", "dr", "dk", "dv"), grads, want):
        assert rel_l2(host(got), ref) <= BF16_REL_L2, name


@pytest.mark.parametrize("B,Hq,Hkv,T,Tkv,d,causal", [(4, 16, 8, 300, 300, 128, True), (2, 8, 4, 200, 333, 64, True),
                                                      (8, 3, 1, 129, 129, 128, False), (1, 16, 16, 260, 260, 128, True)])
def test_backward_pair_counts_that_are_multiples_of_eight(plx, synth, bwd_oracle, B, Hq, Hkv, T, Tkv, d, causal):
    """B * Hkv divisible by 8: the work items take the mapping that deals (batch, kv head) pairs
    over the eight XCDs (the benchmark's launch configuration), here at sizes the oracle covers."""
    _check(plx, synth, bwd_oracle, B, Hq, Hkv, T, Tkv, d, causal, seed=2650 + B + T)
    if causal:  # the sliding-window kernels share the mapping
        _check(plx, synth, bwd_oracle, B, Hq, Hkv, T, Tkv, d, True, seed=2660 + B + T, window=70)


def test_backward_config4_launch_against_the_oracle(plx, synth, bwd_oracle):
    """Benchmark configuration 4 as bench.py launches it (B=4, 16 query / 8 KV heads, T=4096, d=128;
    the pair count takes the XCD mapping and the heavy-blocks-first order): the gradients of two
    (batch, KV head) pairs of THAT launch -- dq, dr of the pair's two query heads, dk, dv of its KV
    head -- against the oracle's, which forms one 4096 x 4096 head at a time."""
    B, Hq, Hkv, T, d = 4, 16, 8, 4096, 128
    y, g = _inputs(synth, B, Hq, Hkv, T, T, d, 2680)
    y["k"] = (y["k"].float() + 0.5 * torch.randn(B, Hkv, 1, d, device=DEV,
                                                 generator=torch.Generator(DEV).manual_seed(2681))).to(torch.bfloat16)
    _, _, _, full = _run(plx, y, g, True)
    for b, hk in ((1, 5), (3, 0)):
        qs, ks = slice(2 * hk, 2 * hk + 2), slice(hk, hk + 1)
        want = bwd_oracle.backward(host(y["q"][b:b + 1, qs]), host(y["r"][b:b + 1, qs]), host(y["k"][b:b + 1, ks]),
                                   host(y["v"][b:b + 1, ks]), host(g[b:b + 1, qs]), y["scale"], causal=True)
        for name, got, ref, hs in zip(("dq", "dr", "dk", "dv"), full, want, (qs, qs, ks, ks)):
            assert_gradient_close(name, host(got[b:b + 1, hs]), ref, BF16_REL_L2, (b, hk))


def test_backward_config4_launch_equals_its_slices(plx, synth):
    """Benchmark configuration 4 as bench.py launches it (B=4, 16 query / 8 KV heads, T=4096, d=128):
    a workgroup's arithmetic does not depend on which work item it is, so the gradients of one
    batch entry and two KV heads' groups must equal, bit for bit, those of a call on just that
    slice (one pair count takes the XCD mapping, the other the plain one; the slice-sized call is
    what test_backward_config4_shape_sampled checks against the oracle)."""
    B, Hq, Hkv, T, d = 4, 16, 8, 4096, 128
    y, g = _inputs(synth, B, Hq, Hkv, T, T, d, 2680)
    o, vbar, stats, full = _run(plx, y, g, True)
    for b, hk0 in ((0, 0), (3, 6), (2, 2)):
        hq0, sl_b = 2 * hk0, slice(b, b + 1)
        sub = {"q": y["q"][sl_b, hq0:hq0 + 4], "r": y["r"][sl_b, hq0:hq0 + 4],
               "k": y["k"][sl_b, hk0:hk0 + 2], "v": y["v"][sl_b, hk0:hk0 + 2], "scale": y["scale"]}
        part = plx.parallax_prefill_backward(sub["q"], sub["r"], sub["k"], sub["v"], o[sl_b, hq0:hq0 + 4],
                                             vbar[sl_b, hq0:hq0 + 4], stats[sl_b, hq0:hq0 + 4].contiguous(),
                                             g[sl_b, hq0:hq0 + 4], y["scale"], causal=True)
        torch.cuda.synchronize()
        for name, got, ref, h0, n in zip(("dq", "dr", "dk", "dv"), part, full, (hq0, hq0, hk0, hk0), (4, 4, 2, 2)):
            assert torch.equal(got, ref[sl_b, h0:h0 + n]), (name, b, hk0)


@pytest.mark.parametrize("B,Hq,Hkv,T,Tkv,d,causal", [(1, 2, 2, 128, 128, 64, True), (2, 4, 2, 77, 77, 32, True),
                                                      (1, 6, 2, 50, 301, 128, True), (2, 4, 4, 130, 257, 16, False),
                                                      (1, 2, 1, 1, 1, 8, True), (1, 2, 2, 300, 300, 256, True)])
def test_backward_fp32_path(plx, synth, bwd_oracle, B, Hq, Hkv, T, Tkv, d, causal):
    """fp32 tensors take the plain kernels: forward row cache and all four gradients to 1e-4."""
    y = synth.prefill_inputs(B, Hq, Hkv, Tkv, d, seed=2700 + T, dtype=torch.float32, device=DEV)
    if Tkv > T:
        y["q"], y["r"] = y["q"][:, :, Tkv - T:].contiguous(), y["r"][:, :, Tkv - T:].contiguous()
    g = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=2701, dtype=torch.float32, device=DEV)["q"].contiguous()
    o, vbar, stats, grads = _run(plx, y, g, causal)
    assert vbar.dtype == torch.float32
    hq, hr, hk, hv = (host(y[n]) for n in "qrkv")
    _, vb, ub, lw = bwd_oracle.forward_with_cache(hq, hr, hk, hv, y["scale"], causal=causal)
    assert max_rel(host(vbar), vb) <= F32_MAX_REL
    np.testing.assert_allclose(host(stats)[..., 0], lw * LOG2E, rtol=0, atol=1e-4)
    assert max_rel(host(stats)[..., 1], ub) <= F32_MAX_REL
    want = bwd_oracle.backward(hq, hr, hk, hv, host(g), y["scale"], causal=causal)
    for name, got, ref in zip(("dq", "dr", "dk", "dv"), grads, want):
        scale = max(np.abs(ref).max(), 1.0)   # dQ = dR = 0 exactly when a row has one key (a - tau cancels)
        assert np.abs(host(got) - ref).max() <= F32_MAX_REL * scale, (name, np.abs(host(got) - ref).max(), scale)


def test_forward_and_backward_in_a_hip_graph(plx, synth):
    """Forward (with the row cache) and backward captured once, replayed with new inputs in the
    captured buffers: every replay equals the eager result bit for bit."""
    import ctypes

    y, g = _inputs(synth, 1, 8, 2, 300, 300, 128, 2800)
    lib = plx.load_library()
    o, vbar = torch.empty_like(y["q"]), torch.empty_like(y["q"])
    stats = torch.empty(y["q"].shape[:3] + (2,), dtype=torch.float32, device=DEV)
    dq, dr = torch.empty_like(y["q"]), torch.empty_like(y["q"])
    dk, dv = torch.empty_like(y["k"]), torch.empty_like(y["k"])
    ws = torch.empty(plx.parallax_prefill_backward_workspace_bytes(1, 8, 300) // 4, dtype=torch.float32,
                     device=DEV)
    fa = plx.prefill_args(y["q"], y["r"], y["k"], y["v"], o, y["scale"], True, True)
    fa.vbar, fa.row_stats = vbar.data_ptr(), stats.data_ptr()
    ba = plx.prefill_bwd_args(y["q"], y["r"], y["k"], y["v"], o, vbar, stats, g, dq, dr, dk, dv, y["scale"],
                              True, ws)
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        cap = int(torch.cuda.current_stream().cuda_stream)
        assert lib.parallax_prefill(ctypes.byref(fa), cap) == 0
        assert lib.parallax_prefill_backward(ctypes.byref(ba), cap) == 0
    torch.cuda.current_stream().wait_stream(side)
    gen = torch.Generator(device=DEV).manual_seed(2801)
    for rep in range(3):
        if rep:
            y["q"].copy_(torch.randn(y["q"].shape, generator=gen, device=DEV))
            g.copy_(torch.randn(g.shape, generator=gen, device=DEV))
        for t in (dq, dr, dk, dv):
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (dq, dr, dk, dv)]
        _, _, _, eager = _run(plx, y, g, True)
        for a, b in zip(got, eager):
            assert torch.equal(a, b)
