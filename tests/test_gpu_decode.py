"""GPU parity of parallax_decode (through the C ABI) against the CPU oracle."""
import numpy as np
import pytest
import torch

from parity import BF16_REL_L2, F32_MAX_REL, host, max_rel, oracle_decode, rel_l2

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def plx():
    from paper_2605_29157_amd import binding

    binding.load_library()  # fails loudly if the HIP library is missing
    assert torch.cuda.is_available()
    return binding


@pytest.fixture(scope="module")
def synth():
    from paper_2605_29157_amd import synth as s

    return s


DEV = "cuda:0"


def _run(plx, x, **kw):
    out = plx.parallax_decode(x["q"], x["r"], x["k"], x["v"], x["scale"],
                              seq_lens=x.get("seq_lens"), **kw)
    torch.cuda.synchronize()
    return host(out)


def test_config2_decode_bf16_full(plx, synth, oracle):
    """benchmark configuration 2: B=8, 16 q heads / 8 kv heads, d=128, L=4096, library split heuristic
    (the launch configuration bench.py times)."""
    x = synth.decode_inputs(8, 16, 8, 4096, 128, seed=1002, device=DEV)
    ref = oracle_decode(oracle, x)
    got = _run(plx, x)
    assert rel_l2(got, ref) <= BF16_REL_L2
    assert max_rel(got, ref) <= 3e-2
    # softmax-only twin == oracle with R = 0
    got0 = _run(plx, x, use_r=False)
    assert rel_l2(got0, oracle_decode(oracle, x, use_r=False)) <= BF16_REL_L2


@pytest.mark.parametrize("L", [1, 2, 15, 16, 31, 32, 33, 127, 128, 129, 511, 1000])
def test_lengths_and_tails(plx, synth, oracle, L):
    x = synth.decode_inputs(2, 4, 2, L, 128, seed=200 + L, device=DEV)
    ref = oracle_decode(oracle, x)
    for S in (0, 1, 3):
        got = _run(plx, x, num_splits=S)
        assert rel_l2(got, ref) <= BF16_REL_L2, (L, S)
    if L == 1:  # one key: the output is that value row exactly (bf16 in, bf16 out)
        v = host(x["v"])[:, :, 0, :]
        np.testing.assert_array_equal(_run(plx, x, num_splits=1), np.repeat(v, 2, axis=1))


@pytest.mark.parametrize("S", [1, 2, 5, 16, 128])
def test_split_counts_agree_incl_empty_splits(plx, synth, oracle, S):
    x = synth.decode_inputs(3, 8, 4, 1500, 128, seed=31, device=DEV, ragged=True)
    ref = oracle_decode(oracle, x)
    got = _run(plx, x, num_splits=S)  # S=128 leaves most splits empty
    assert rel_l2(got, ref) <= BF16_REL_L2


def test_ragged_with_zero_length_sequence(plx, synth, oracle):
    x = synth.decode_inputs(4, 4, 2, 700, 128, seed=41, device=DEV, ragged=True)
    x["seq_lens"][1] = 0
    x["seq_lens"][2] = 1
    ref = oracle_decode(oracle, x)
    for S in (1, 4):
        got = _run(plx, x, num_splits=S)
        assert np.all(got[1] == 0.0)  # documented reading of the empty key set
        keep = [0, 2, 3]
        assert rel_l2(got[keep], ref[keep]) <= BF16_REL_L2


@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (8, 2), (8, 1), (6, 2), (12, 1), (16, 1), (32, 2)])
def test_gqa_group_sizes(plx, synth, oracle, Hq, Hkv):
    x = synth.decode_inputs(2, Hq, Hkv, 300, 128, seed=50 + Hq, device=DEV)
    ref = oracle_decode(oracle, x)
    got = _run(plx, x, num_splits=2)
    assert rel_l2(got, ref) <= BF16_REL_L2


def test_head_dim_64(plx, synth, oracle):
    x = synth.decode_inputs(3, 8, 4, 777, 64, seed=64, device=DEV, ragged=True)
    ref = oracle_decode(oracle, x)
    for S in (1, 4):
        assert rel_l2(_run(plx, x, num_splits=S), ref) <= BF16_REL_L2


def test_strided_cache_layout(plx, synth, oracle):
    """K/V stored as [B, L, Hkv, d] and passed as a permuted view (row stride = Hkv*d)."""
    x = synth.decode_inputs(2, 4, 2, 400, 128, seed=71, device=DEV)
    ref = oracle_decode(oracle, x)
    xs = dict(x)
    xs["k"] = x["k"].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    xs["v"] = x["v"].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert xs["k"].stride(2) == 2 * 128
    assert rel_l2(_run(plx, xs, num_splits=2), ref) <= BF16_REL_L2


def test_key_offset_and_small_probe(plx, synth, oracle):
    """Keys with a common offset (the correction must centre them) and a probe scaled by 0.1."""
    x = synth.decode_inputs(2, 16, 8, 2048, 128, seed=81, device=DEV, r_scale=0.1)
    off = torch.randn(2, 8, 1, 128, device=DEV, generator=torch.Generator(DEV).manual_seed(5))
    x["k"] = (x["k"].float() + 0.5 * off).to(torch.bfloat16)
    ref = oracle_decode(oracle, x)
    assert rel_l2(_run(plx, x), ref) <= BF16_REL_L2


def test_large_logit_range_and_zero_scale(plx, synth, oracle):
    x = synth.decode_inputs(2, 4, 2, 900, 128, seed=85, device=DEV)
    x["q"] = (x["q"].float() * 40.0).to(torch.bfloat16)
    ref = oracle_decode(oracle, x)
    got = _run(plx, x, num_splits=3)
    assert np.isfinite(got).all() and rel_l2(got, ref) <= BF16_REL_L2
    x = synth.decode_inputs(2, 4, 2, 900, 128, seed=86, device=DEV, r_scale=0.2)
    x["scale"] = 0.0
    assert rel_l2(_run(plx, x, num_splits=3), oracle_decode(oracle, x)) <= BF16_REL_L2


def test_deterministic_run_to_run(plx, synth):
    x = synth.decode_inputs(4, 16, 8, 3000, 128, seed=91, device=DEV, ragged=True)
    a = _run(plx, x, num_splits=8)
    b = _run(plx, x, num_splits=8)
    np.testing.assert_array_equal(a, b)


@pytest.mark.parametrize("page_size", [1, 16, 48, 128, 256])
def test_paged_cache_matches_contiguous(plx, synth, oracle, page_size):
    """Paged KV cache: same keys behind a block table in a shuffled page pool. The kernel must
    return bit-for-bit what it returns on the contiguous cache (same tiles, same order), and
    that agrees with the oracle."""
    x = synth.decode_inputs(3, 16, 8, 1500, 128, seed=95, device=DEV, ragged=True)
    kp, vp, table = synth.paged_cache(x, page_size, seed=96)
    ref = _run(plx, x, num_splits=4)
    out = plx.parallax_decode(x["q"], x["r"], kp, vp, x["scale"], seq_lens=x["seq_lens"],
                              num_splits=4, block_table=table, max_len=1500)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(out), ref)
    assert rel_l2(ref, oracle_decode(oracle, x)) <= BF16_REL_L2


def test_paged_cache_other_layouts(plx, synth, oracle):
    # d = 64, softmax-only twin, heuristic split count, fp32 path
    x = synth.decode_inputs(2, 8, 4, 700, 64, seed=97, device=DEV, ragged=True)
    kp, vp, table = synth.paged_cache(x, 32, seed=98)
    out = plx.parallax_decode(x["q"], x["r"], kp, vp, x["scale"], seq_lens=x["seq_lens"],
                              block_table=table, max_len=700)
    twin = plx.parallax_decode(x["q"], None, kp, vp, x["scale"], seq_lens=x["seq_lens"],
                               use_r=False, block_table=table, max_len=700)
    torch.cuda.synchronize()
    assert rel_l2(host(out), oracle_decode(oracle, x)) <= BF16_REL_L2
    assert rel_l2(host(twin), oracle_decode(oracle, x, use_r=False)) <= BF16_REL_L2
    x = synth.decode_inputs(2, 4, 2, 300, 64, seed=99, dtype=torch.float32, device=DEV, ragged=True)
    kp, vp, table = synth.paged_cache(x, 16, seed=100)
    out = plx.parallax_decode(x["q"], x["r"], kp, vp, x["scale"], seq_lens=x["seq_lens"],
                              block_table=table, max_len=300)
    torch.cuda.synchronize()
    assert max_rel(host(out), oracle_decode(oracle, x)) <= F32_MAX_REL


def _multirow_inputs(synth, B, Hq, Hkv, L, d, Tq, seed, dtype=torch.bfloat16, lens=None):
    """Decode inputs whose q, r hold Tq rows per head: [B, Hq, Tq, d]."""
    x = synth.decode_inputs(B, Hq, Hkv, L, d, seed=seed, dtype=dtype, device=DEV)
    more = synth.prefill_inputs(B, Hq, Hkv, Tq, d, seed=seed + 1, dtype=dtype, device=DEV)
    x["q"], x["r"] = more["q"].contiguous(), more["r"].contiguous()
    if lens is not None:
        x["seq_lens"] = torch.tensor(lens, dtype=torch.int32, device=DEV)
    return x


def _multirow_oracle(oracle, x, use_r=True, window=0):
    """Row t of the Tq rows is position L_b - Tq + t: causal chunk over the first L_b keys."""
    q, r, k, v = (host(x[n]) for n in "qrkv")
    B, Hq, Tq, d = q.shape
    lens = host(x["seq_lens"]).astype(int) if x.get("seq_lens") is not None else [k.shape[2]] * B
    out = np.zeros((B, Hq, Tq, d))
    for b in range(B):
        Lb = int(lens[b])
        t0 = max(0, Tq - Lb)  # rows before position 0 see nothing: zeros
        if Lb == 0:
            continue
        rr = r[b:b + 1, :, t0:] if use_r else np.zeros_like(r[b:b + 1, :, t0:])
        out[b, :, t0:] = oracle.forward(q[b:b + 1, :, t0:], rr, k[b:b + 1, :, :Lb], v[b:b + 1, :, :Lb],
                                        x["scale"], causal=True, window=window)[0]
    return out


@pytest.mark.parametrize("Hq,Hkv,Tq", [(16, 8, 2), (16, 8, 5), (16, 8, 8), (4, 4, 16), (8, 1, 2),
                                       (8, 2, 4), (6, 2, 3)])
@pytest.mark.parametrize("S", [0, 1, 5])
def test_several_query_rows_per_sequence(plx, synth, oracle, Hq, Hkv, Tq, S):
    """Tq query rows as extra MFMA columns: the rows are the last Tq positions (speculative rows)."""
    lens = [1500, 3, 777, 1][:3] if S else [1500, 1024, 129]
    x = _multirow_inputs(synth, 3, Hq, Hkv, 1500, 128, Tq, seed=400 + Tq + Hq, lens=lens)
    ref = _multirow_oracle(oracle, x)
    out = plx.parallax_decode(x["q"], x["r"], x["k"], x["v"], x["scale"], seq_lens=x["seq_lens"],
                              num_splits=S)
    torch.cuda.synchronize()
    got = host(out)
    assert got.shape == ref.shape and np.isfinite(got).all()
    assert rel_l2(got, ref) <= BF16_REL_L2, (Hq, Hkv, Tq, S)
    row_err = np.linalg.norm(got - ref, axis=-1) / np.maximum(np.linalg.norm(ref, axis=-1), 1e-6)
    assert row_err.max() <= 5 * BF16_REL_L2, (Hq, Hkv, Tq, S, np.unravel_index(row_err.argmax(), row_err.shape))


def test_several_query_rows_other_paths(plx, synth, oracle):
    # one row given as [B, Hq, 1, d] is the ordinary decode step, bit for bit
    x = synth.decode_inputs(2, 16, 8, 900, 128, seed=420, device=DEV, ragged=True)
    a = _run(plx, x, num_splits=3)
    b4 = plx.parallax_decode(x["q"][:, :, None].contiguous(), x["r"][:, :, None].contiguous(), x["k"],
                             x["v"], x["scale"], seq_lens=x["seq_lens"], num_splits=3)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(b4)[:, :, 0], a)
    # the same rows through the prefill kernel (chunked causal): two kernels, one operator
    y = _multirow_inputs(synth, 2, 16, 8, 640, 128, 6, seed=421)
    dec = plx.parallax_decode(y["q"], y["r"], y["k"], y["v"], y["scale"])
    pre = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=True)
    torch.cuda.synchronize()
    assert rel_l2(host(dec), host(pre)) <= BF16_REL_L2
    # rows that sit before position 0 (sequence shorter than Tq) come out as zeros
    z = _multirow_inputs(synth, 2, 16, 8, 256, 128, 4, seed=422, lens=[2, 256])
    got = host(plx.parallax_decode(z["q"], z["r"], z["k"], z["v"], z["scale"], seq_lens=z["seq_lens"]))
    torch.cuda.synchronize()
    assert (got[0, :, :2] == 0).all() and rel_l2(got, _multirow_oracle(oracle, z)) <= BF16_REL_L2
    # d = 64, softmax-only twin, paged cache, fp32
    w = _multirow_inputs(synth, 2, 8, 4, 500, 64, 3, seed=423, lens=[500, 77])
    kp, vp, table = synth.paged_cache(w, 16, seed=424)
    got = plx.parallax_decode(w["q"], None, kp, vp, w["scale"], seq_lens=w["seq_lens"], use_r=False,
                              block_table=table, max_len=500)
    torch.cuda.synchronize()
    assert rel_l2(host(got), _multirow_oracle(oracle, w, use_r=False)) <= BF16_REL_L2
    f = _multirow_inputs(synth, 2, 4, 2, 200, 64, 20, seed=425, dtype=torch.float32, lens=[200, 31])
    got = plx.parallax_decode(f["q"], f["r"], f["k"], f["v"], f["scale"], seq_lens=f["seq_lens"])
    torch.cuda.synchronize()
    assert max_rel(host(got), _multirow_oracle(oracle, f)) <= F32_MAX_REL
    # a GQA group of more than 16 heads is not supported by the bf16 kernels
    bad = _multirow_inputs(synth, 1, 34, 2, 256, 128, 1, seed=426)
    with pytest.raises(plx.ParallaxError):
        plx.parallax_decode(bad["q"], bad["r"], bad["k"], bad["v"], bad["scale"])


@pytest.mark.parametrize("Hq,Hkv,Tq", [(16, 8, 9), (16, 8, 20), (8, 2, 7), (8, 1, 5), (6, 2, 11), (8, 8, 40), (16, 1, 3), (24, 2, 2)])
@pytest.mark.parametrize("S", [0, 1, 4])
def test_more_columns_than_one_launch_holds(plx, synth, oracle, Hq, Hkv, Tq, S):
    """(heads of a group) x (query rows) > 16: one launch per 16 / G rows over the same cache and
    workspace, one combine; every launch sees the sequence up to its own last row."""
    lens = [900, 5, 333]
    x = _multirow_inputs(synth, 3, Hq, Hkv, 900, 128, Tq, seed=430 + Tq + Hq, lens=lens)
    ref = _multirow_oracle(oracle, x)
    out = plx.parallax_decode(x["q"], x["r"], x["k"], x["v"], x["scale"], seq_lens=x["seq_lens"], num_splits=S)
    torch.cuda.synchronize()
    got = host(out)
    assert np.isfinite(got).all() and rel_l2(got, ref) <= BF16_REL_L2, (Hq, Hkv, Tq, S)
    row_err = np.linalg.norm(got - ref, axis=-1) / np.maximum(np.linalg.norm(ref, axis=-1), 1e-6)
    assert row_err.max() <= 5 * BF16_REL_L2, (Hq, Hkv, Tq, S, np.unravel_index(row_err.argmax(), row_err.shape))
    if S == 4:   # the in-kernel reduction and a sliding window take the same passes
        cnt = torch.zeros(3 * Hkv, dtype=torch.int32, device=DEV)
        fused = plx.parallax_decode_fused(x["q"], x["r"], x["k"], x["v"], x["scale"], cnt, seq_lens=x["seq_lens"],
                                          num_splits=S)
        torch.cuda.synchronize()
        assert torch.equal(fused, out) and int(cnt.abs().sum()) == 0
        win = plx.parallax_decode(x["q"], x["r"], x["k"], x["v"], x["scale"], seq_lens=x["seq_lens"], num_splits=S,
                                  window=100)
        torch.cuda.synchronize()
        wref = _multirow_oracle(oracle, x, window=100)
        assert rel_l2(host(win), wref) <= BF16_REL_L2


def test_two_streams_with_their_own_workspaces(plx, synth):
    """The library keeps no state: launches on different streams, each with its own workspace and
    output, interleave freely and return what the same calls return alone."""
    xs = [synth.decode_inputs(4, 16, 8, 6000, 128, seed=430 + i, device=DEV, ragged=True) for i in range(2)]
    ys = [synth.prefill_inputs(1, 16, 8, 700, 128, seed=440 + i, device=DEV) for i in range(2)]
    alone_d = [_run(plx, x, num_splits=8) for x in xs]
    alone_p = [host(plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"])) for y in ys]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ws = [torch.empty(plx.parallax_decode_workspace_bytes(4, 16, 8, 6000, 128) // 4,
                      dtype=torch.float32, device=DEV) for _ in range(2)]
    out_d = [torch.empty_like(x["q"]) for x in xs]
    out_p = [torch.empty_like(y["q"]) for y in ys]
    for s_ in streams:
        s_.wait_stream(torch.cuda.current_stream())
    for rep in range(5):
        for i, s_ in enumerate(streams):
            plx.parallax_decode(xs[i]["q"], xs[i]["r"], xs[i]["k"], xs[i]["v"], xs[i]["scale"],
                                seq_lens=xs[i]["seq_lens"], num_splits=8, workspace=ws[i],
                                out=out_d[i], stream=s_)
            plx.parallax_prefill(ys[i]["q"], ys[i]["r"], ys[i]["k"], ys[i]["v"], ys[i]["scale"],
                                 out=out_p[i], stream=s_)
    torch.cuda.synchronize()
    for i in range(2):
        np.testing.assert_array_equal(host(out_d[i]), alone_d[i])
        np.testing.assert_array_equal(host(out_p[i]), alone_p[i])


def test_hip_graph_replays_match_eager(plx, synth, oracle):
    """Decode and prefill captured in one HIP graph: every replay, with eager work and
    synchronisation in between and inputs changed in place, equals the eager result."""
    x = synth.decode_inputs(4, 16, 8, 2500, 128, seed=92, device=DEV, ragged=True)
    y = synth.prefill_inputs(1, 4, 2, 300, 128, seed=93, device=DEV)
    B, Hq, d = x["q"].shape
    ws = torch.empty(plx.parallax_decode_workspace_bytes(B, Hq, 8, 2500, d) // 4,
                     dtype=torch.float32, device=DEV)
    out_d, out_p = torch.empty_like(x["q"]), torch.empty_like(y["q"])
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        cap = torch.cuda.current_stream()
        plx.parallax_decode(x["q"], x["r"], x["k"], x["v"], x["scale"], seq_lens=x["seq_lens"],
                            workspace=ws, out=out_d, stream=cap)
        plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=True, out=out_p,
                             stream=cap)
    torch.cuda.current_stream().wait_stream(side)
    gen = torch.Generator(device=DEV).manual_seed(94)
    for rep in range(4):
        if rep:  # new inputs in the captured buffers
            x["q"].copy_(torch.randn(x["q"].shape, generator=gen, device=DEV))
            y["r"].copy_(torch.randn(y["r"].shape, generator=gen, device=DEV))
        out_d.zero_()
        out_p.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got_d, got_p = host(out_d), host(out_p)
        eager_d = _run(plx, x, workspace=ws)
        eager_p = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=True)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(got_d, eager_d)
        np.testing.assert_array_equal(got_p, host(eager_p))
    assert rel_l2(got_d, oracle_decode(oracle, x)) <= BF16_REL_L2


def test_workspace_partials_match_streaming_form(plx, synth):
    """The split workspace holds, per split, the unnormalised state of Algorithm 1 over that
    split's key range. Compare what is unique: log-sum-exp m + log2 d1, d2/d1, O1/d1, O2/d1."""
    from oracle import forms

    B, Hq, Hkv, L, d, S = 1, 4, 2, 1024, 128, 4
    x = synth.decode_inputs(B, Hq, Hkv, L, d, seed=101, device=DEV)
    ws = torch.zeros(B * Hq * S * (2 * d + 4), dtype=torch.float32, device=DEV)
    plx.parallax_decode(x["q"], x["r"], x["k"], x["v"], x["scale"], num_splits=S, workspace=ws)
    torch.cuda.synchronize()
    rec = ws.cpu().numpy().reshape(B, Hq, S, 2 * d + 4).astype(np.float64)
    q, r, k, v = (host(x[n]).astype(np.float64) for n in "qrkv")
    per = L // S  # 8 block tiles of 128 keys, two per split
    for h in range(Hq):
        for s in range(S):
            m, d1, d2, O1, O2 = forms.streaming_partial(q[0, h][None], r[0, h][None], k[0, h // 2],
                                                        v[0, h // 2], x["scale"], 32,
                                                        s * per, (s + 1) * per)
            g = rec[0, h, s]
            assert abs((g[0] + np.log2(g[1])) - (m[0] + np.log2(d1[0]))) < 2e-3
            assert abs(g[2] / g[1] - d2[0] / d1[0]) < 2e-2 * max(1.0, abs(d2[0] / d1[0]))
            assert rel_l2(g[4:4 + d] / g[1], O1[0] / d1[0]) < BF16_REL_L2
            assert rel_l2(g[4 + d:] / g[1], O2[0] / d1[0]) < BF16_REL_L2


def test_partials_then_combine_equals_decode(plx, synth):
    """The two exported halves chained by the caller give bit-identical output to the fused
    entry point, also for S = 1 (where the fused call skips the workspace)."""
    x = synth.decode_inputs(3, 8, 4, 900, 128, seed=105, device=DEV, ragged=True)
    for S in (1, 6):
        ws = torch.empty(3 * 8 * S * 260, dtype=torch.float32, device=DEV)
        plx.parallax_decode_partials(x["q"], x["r"], x["k"], x["v"], x["scale"], S, ws,
                                     seq_lens=x["seq_lens"])
        out = torch.empty_like(x["q"])
        plx.parallax_decode_combine(ws, out, 4, S)
        torch.cuda.synchronize()
        fused = _run(plx, x, num_splits=S)
        if S > 1:
            np.testing.assert_array_equal(host(out), fused)
        else:
            assert rel_l2(host(out), fused.astype(np.float64)) < 1e-6 + 4e-3


def test_decode_fp32_path(plx, synth, oracle):
    x = synth.decode_inputs(2, 4, 2, 700, 64, seed=111, dtype=torch.float32, device=DEV, ragged=True)
    ref = oracle_decode(oracle, x)
    got = _run(plx, x)
    assert max_rel(got, ref) <= F32_MAX_REL


def test_errors_surface_as_exceptions(plx, synth):
    x = synth.decode_inputs(1, 4, 2, 64, 128, seed=1, device=DEV)
    with pytest.raises(plx.ParallaxError) as e:
        plx.parallax_decode(x["q"], x["r"], x["k"], x["v"], x["scale"], num_splits=4,
                            workspace=torch.empty(8, dtype=torch.float32, device=DEV))
    assert e.value.status == plx.PLX_ERR_WORKSPACE


def _sampled_sequences(B, lens):
    lens = lens.cpu().numpy()
    picks = {int(np.argmin(lens)), int(np.argmax(lens)), 1 % B, B - 1}
    return sorted(picks)


@pytest.mark.parametrize("B,L,ragged", [(1, 1024, False), (1, 1024, True), (1, 65536, False), (1, 65536, True),
                                        (16, 4096, True), (64, 16384, True), (128, 1024, True), (128, 65536, True)])
def test_config3_sweep_corners_sampled(plx, synth, oracle, B, L, ragged):
    """Corners (and the middle) of the config-3 grid, B in {1, 16, 64, 128} x L in {1k, 4k, 16k,
    64k}, at 16 query / 8 KV heads, d = 128, lengths uniform on [L/2, L], with the library's own
    split count -- the launches bench.py times; the branches of the split heuristic differ over the
    grid (B=1: 64 / 4 short splits; B=16: by pairs; B >= 64: by length only; B=128 x 64k: 17 GB per
    tensor, offsets beyond 2^31 elements). Oracle on all heads of up to four sequences: shortest,
    longest, two more."""
    x = synth.decode_inputs(B, 16, 8, L, 128, seed=1003 + B + L, device=DEV, ragged=ragged)
    got = _run(plx, x)
    assert np.isfinite(got).all()
    lens = x["seq_lens"] if ragged else torch.full((B,), L)
    seqs = _sampled_sequences(B, lens)
    ref = oracle_decode(oracle, x, seqs=seqs)
    assert rel_l2(got[seqs], ref) <= BF16_REL_L2, (B, L, seqs)
    per_seq = [rel_l2(got[s], ref[i]) for i, s in enumerate(seqs)]
    assert max(per_seq) <= BF16_REL_L2, (B, L, seqs, per_seq)


def test_config5b_long_context_sampled(plx, synth, oracle):
    """Config 5 part two: B=32, KV length 131072, probe scaled by 0.1 (K and V are 8.6 GB each,
    offsets beyond 2^31 elements); oracle on 3 sampled sequences."""
    x = synth.decode_inputs(32, 16, 8, 131072, 128, seed=1005, device=DEV, r_scale=0.1)
    got = _run(plx, x)
    seqs = [0, 17, 31]
    ref = oracle_decode(oracle, x, seqs=seqs)
    assert rel_l2(got[seqs], ref) <= BF16_REL_L2
    assert np.isfinite(got).all()


def test_block_sparse_decode_is_a_block_table_of_selected_pages(plx, synth, oracle):
    """Block-sparse decode needs no kernel of its own: a block table that lists only the selected
    pages of a sequence (any order is fine for a single query row -- the sum over keys does not
    depend on it) is attention over exactly those keys. Checked against the oracle on the
    gathered keys."""
    page = 64
    x = synth.decode_inputs(3, 16, 8, 2048, 128, seed=130, device=DEV)
    kp, vp, table = synth.paged_cache(x, page, seed=131)
    rng = np.random.default_rng(132)
    keep = [np.sort(rng.choice(2048 // page, size=n, replace=False)) for n in (5, 17, 32)]
    width = max(len(s) for s in keep)
    sel = torch.zeros((3, width), dtype=torch.int32, device=DEV)
    for b, s in enumerate(keep):
        sel[b, :len(s)] = table[b, torch.as_tensor(s, device=DEV)]
    lens = torch.tensor([len(s) * page for s in keep], dtype=torch.int32, device=DEV)
    out = plx.parallax_decode(x["q"], x["r"], kp, vp, x["scale"], seq_lens=lens, block_table=sel,
                              max_len=width * page)
    torch.cuda.synchronize()
    q, r, k, v = (host(x[n]) for n in "qrkv")
    for b, s in enumerate(keep):
        cols = np.concatenate([np.arange(p * page, (p + 1) * page) for p in s])
        ref = oracle.forward(q[b:b + 1, :, None], r[b:b + 1, :, None], k[b:b + 1][:, :, cols],
                             v[b:b + 1][:, :, cols], x["scale"])[0, :, 0]
        assert rel_l2(host(out)[b], ref) <= BF16_REL_L2, b
