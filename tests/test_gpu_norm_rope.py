"""GPU parity of parallax_norm_rope (RMSNorm + RoPE on q, rho, k in one launch, through the C ABI)
against the float64 oracle, alone and in front of the attention kernels."""
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
def nr():
    from oracle import norm_rope

    return norm_rope


def _rand(shape, seed, dtype):
    g = torch.Generator(device=DEV).manual_seed(seed)
    return (torch.randn(shape, generator=g, device=DEV) * 1.7).to(dtype)


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.bfloat16, 64), (torch.float32, 128),
                                     (torch.float32, 16), (torch.float32, 256), (torch.float32, 64)])
def test_three_tensors_one_launch(plx, nr, dtype, d):
    B, T = 3, 37
    q, r, k = _rand((B, 6, T, d), 1, dtype), _rand((B, 6, T, d), 2, dtype), _rand((B, 2, T, d), 3, dtype)
    gq, gr, gk = (1.0 + 0.3 * _rand((d,), 4 + i, torch.float32) for i in range(3))
    pos0 = torch.tensor([0, 4090, 131000], dtype=torch.int32, device=DEV)
    oq, orr, ok = plx.parallax_norm_rope([(q, gq, True), (r, gr, False), (k, gk, True)], pos0=pos0,
                                         eps=1e-6, theta=1.0e6)
    torch.cuda.synchronize()
    pos = host(pos0)[:, None, None] + np.arange(T)[None, None, :]
    want = [nr.norm_rope(host(q), host(gq), pos), nr.rms_norm(host(r), host(gr)), nr.norm_rope(host(k), host(gk), pos)]
    for got, ref in zip((oq, orr, ok), want):
        assert got.dtype == dtype and np.isfinite(host(got)).all()
        if dtype == torch.float32:
            assert max_rel(host(got), ref) <= F32_MAX_REL
        else:
            assert rel_l2(host(got), ref) <= BF16_REL_L2


def test_in_place_one_tensor_defaults_and_odd_sizes(plx, nr):
    x = _rand((1, 1, 1, 64), 10, torch.float32)
    g = torch.ones(64, dtype=torch.float32, device=DEV)
    ref = nr.norm_rope(host(x), host(g), np.zeros((1, 1, 1)))
    (y,) = plx.parallax_norm_rope([(x, g, True)], inplace=True)
    torch.cuda.synchronize()
    assert y.data_ptr() == x.data_ptr()
    assert max_rel(host(x), ref) <= F32_MAX_REL            # position 0: the norm alone
    np.testing.assert_allclose((host(x) ** 2).mean(), 1.0, rtol=1e-4)
    # many rows, not a multiple of the rows a workgroup takes
    x = _rand((2, 5, 333, 128), 11, torch.bfloat16)
    g = 1.0 + 0.1 * _rand((128,), 12, torch.float32)
    (y,) = plx.parallax_norm_rope([(x, g, True)], theta=1.0e4, eps=1e-5)
    torch.cuda.synchronize()
    ref = nr.norm_rope(host(x), host(g), np.arange(333)[None, None, :], eps=1e-5, theta=1.0e4)
    assert rel_l2(host(y), ref) <= BF16_REL_L2


def test_prepared_tensors_feed_the_attention_kernels(plx, nr, oracle):
    """Raw projections -> parallax_norm_rope -> parallax_prefill / parallax_decode against the
    oracle chain (norm + rope in float64 on the same raw values, rounded to bf16 where the
    kernels round, then the attention oracle)."""
    from paper_2605_29157_amd import synth

    B, Hq, Hkv, T, d = 2, 8, 4, 200, 128
    y = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=20, device=DEV)
    gq, gr, gk = (1.0 + 0.2 * _rand((d,), 21 + i, torch.float32) for i in range(3))
    q2, r2, k2 = plx.parallax_norm_rope([(y["q"], gq, True), (y["r"], gr, True), (y["k"], gk, True)])
    out = plx.parallax_prefill(q2, r2, k2, y["v"], y["scale"], causal=True)
    torch.cuda.synchronize()
    pos = np.arange(T)[None, None, :]
    as_bf16 = lambda a: torch.tensor(a).to(torch.bfloat16).float().numpy()
    qo, ro, ko = (as_bf16(nr.norm_rope(host(y[n]), host(g), pos)) for n, g in (("q", gq), ("r", gr), ("k", gk)))
    # the kernel's bf16 outputs may differ from the rounded oracle by one bf16 step here and there
    assert rel_l2(host(q2), qo) <= 3e-3 and rel_l2(host(k2), ko) <= 3e-3
    ref = oracle.forward(host(q2), host(r2), host(k2), host(y["v"]), y["scale"], causal=True)
    assert rel_l2(host(out), ref) <= BF16_REL_L2
    ref_chain = oracle.forward(qo, ro, ko, host(y["v"]), y["scale"], causal=True)
    assert rel_l2(host(out), ref_chain) <= BF16_REL_L2
    # decode step: the last row's q, rho at position T - 1 over the prepared cache
    qd, rd = y["q"][:, :, T - 1:].contiguous(), y["r"][:, :, T - 1:].contiguous()
    pos0 = torch.full((B,), T - 1, dtype=torch.int32, device=DEV)
    q1, r1 = plx.parallax_norm_rope([(qd, gq, True), (rd, gr, True)], pos0=pos0)
    dec = plx.parallax_decode(q1[:, :, 0].contiguous(), r1[:, :, 0].contiguous(), k2, y["v"], y["scale"])
    torch.cuda.synchronize()
    assert rel_l2(host(dec), host(out)[:, :, T - 1]) <= BF16_REL_L2


def test_norm_rope_rejects_bad_arguments(plx):
    x = _rand((1, 2, 4, 128), 30, torch.bfloat16)
    g = torch.ones(128, dtype=torch.float32, device=DEV)
    with pytest.raises(plx.ParallaxError):
        plx.parallax_norm_rope([(x, g, True)], theta=1.0)
    with pytest.raises(plx.ParallaxError):
        plx.parallax_norm_rope([(x, g, True)], eps=-1.0)
    with pytest.raises(plx.ParallaxError):
        plx.parallax_norm_rope([(_rand((1, 2, 4, 96), 31, torch.bfloat16), torch.ones(96, device=DEV), True)])


def test_rope_table_against_the_definition(plx):
    """(cos, sin) of pos * theta^(-2i/d), angles up to 1.3e5 radians."""
    for d, theta, n_pos in ((128, 1.0e6, 4100), (64, 1.0e4, 700)):
        tab = plx.parallax_rope_table(n_pos, d, theta, device=DEV)
        far = plx.parallax_rope_table(131072, d, theta, device=DEV)[-3:]
        torch.cuda.synchronize()
        for t, pos in ((tab, np.arange(n_pos)), (far, np.arange(131069, 131072))):
            ang = pos[:, None].astype(np.float64) * theta ** (-np.arange(0, d, 2, dtype=np.float64) / d)
            got = host(t).astype(np.float64)
            np.testing.assert_allclose(got[..., 0], np.cos(ang), rtol=0, atol=3e-6)
            np.testing.assert_allclose(got[..., 1], np.sin(ang), rtol=0, atol=3e-6)


@pytest.mark.parametrize("d,T,Tkv,causal,rope_r", [(128, 300, 300, True, True), (128, 200, 517, True, False),
                                                   (64, 513, 513, True, True), (64, 77, 300, False, True),
                                                   (128, 129, 129, False, False)])
def test_prefill_prepares_q_and_rho_itself(plx, nr, oracle, d, T, Tkv, causal, rope_r):
    """RMSNorm + RoPE on q, rho inside the prefill kernel: against the two-launch chain
    (parallax_norm_rope, then parallax_prefill on its outputs) and against the oracle chain, with
    the chunk's rows at positions behind a cache (pos0 = Tkv - T plus a per-sequence offset)."""
    from paper_2605_29157_amd import synth

    B, Hq, Hkv = 2, 8, 4
    y = synth.prefill_inputs(B, Hq, Hkv, Tkv, d, seed=40 + T, device=DEV)
    q, r = y["q"][:, :, Tkv - T:].contiguous(), y["r"][:, :, Tkv - T:].contiguous()
    gq, gr, gk = (1.0 + 0.2 * _rand((d,), 41 + i, torch.float32) for i in range(3))
    kpos0 = torch.tensor([0, 1000], dtype=torch.int32, device=DEV)
    qpos0 = kpos0 + (Tkv - T)
    (k2,) = plx.parallax_norm_rope([(y["k"], gk, True)], pos0=kpos0)
    table = plx.parallax_rope_table(1000 + Tkv, d, device=DEV)
    prep = plx.qr_prep(gq, gr, table, qpos0, rope_q=True, rope_r=rope_r)
    fused = plx.parallax_prefill(q, r, k2, y["v"], y["scale"], causal=causal, prep=prep)
    q2, r2 = plx.parallax_norm_rope([(q, gq, True), (r, gr, rope_r)], pos0=qpos0)
    chain = plx.parallax_prefill(q2, r2, k2, y["v"], y["scale"], causal=causal)
    torch.cuda.synchronize()
    # the same mathematics with the roundings to bf16 at other places (the kernel leaves the
    # 1 / rms factors out of the stored rows and applies them to the scores and to O2, d2)
    assert rel_l2(host(fused), host(chain).astype(np.float64)) <= 5e-3
    # oracle chain: norm + rope in float64 on the raw values, then the attention oracle
    pos_q = (host(qpos0)[:, None, None] + np.arange(T)[None, None, :])
    pos_k = (host(kpos0)[:, None, None] + np.arange(Tkv)[None, None, :])
    qo = nr.norm_rope(host(q), host(gq), pos_q)
    ro = nr.norm_rope(host(r), host(gr), pos_q) if rope_r else nr.rms_norm(host(r), host(gr))
    ko = nr.norm_rope(host(y["k"]), host(gk), pos_k)
    ref = oracle.forward(qo, ro, ko, host(y["v"]), y["scale"], causal=causal)
    assert rel_l2(host(fused), ref) <= BF16_REL_L2
    # RMSNorm alone (no table)
    prep_n = plx.qr_prep(gq, gr, None, None)
    fused_n = plx.parallax_prefill(q, r, k2, y["v"], y["scale"], causal=causal, prep=prep_n)
    ref_n = oracle.forward(nr.rms_norm(host(q), host(gq)), nr.rms_norm(host(r), host(gr)), host(k2), host(y["v"]),
                           y["scale"], causal=causal)
    assert rel_l2(host(fused_n), ref_n) <= BF16_REL_L2


@pytest.mark.parametrize("d,Tq,S,paged", [(128, 1, 0, False), (128, 3, 4, False), (64, 1, 3, False), (128, 1, 2, True),
                                          (128, 9, 3, False)])
def test_decode_prepares_q_and_rho_itself(plx, nr, oracle, d, Tq, S, paged):
    """The decode rows are the last Tq positions of each (ragged) sequence: their q, rho are
    normalised and rotated in the split kernel, against the two-launch chain and the oracle chain."""
    from paper_2605_29157_amd import synth

    B, Hq, Hkv, L = 3, 8, 4, 700
    x = synth.decode_inputs(B, Hq, Hkv, L, d, seed=50 + Tq, device=DEV, ragged=True)
    q = _rand((B, Hq, Tq, d), 51, torch.bfloat16)
    r = _rand((B, Hq, Tq, d), 52, torch.bfloat16)
    gq, gr = (1.0 + 0.2 * _rand((d,), 53 + i, torch.float32) for i in range(2))
    table = plx.parallax_rope_table(L, d, device=DEV)
    prep = plx.qr_prep(gq, gr, table, None)
    kw = {}
    k, v = x["k"], x["v"]
    if paged:
        k, v, tb = synth.paged_cache(x, 48, seed=55)
        kw = dict(block_table=tb, max_len=L)
    qa, ra = (q, r) if Tq > 1 else (q[:, :, 0].contiguous(), r[:, :, 0].contiguous())
    fused = plx.parallax_decode(qa, ra, k, v, x["scale"], seq_lens=x["seq_lens"], num_splits=S, prep=prep, **kw)
    pos0 = (x["seq_lens"] - Tq).to(torch.int32)
    q2, r2 = plx.parallax_norm_rope([(q, gq, True), (r, gr, True)], pos0=pos0)
    q2a, r2a = (q2, r2) if Tq > 1 else (q2[:, :, 0].contiguous(), r2[:, :, 0].contiguous())
    chain = plx.parallax_decode(q2a, r2a, k, v, x["scale"], seq_lens=x["seq_lens"], num_splits=S, **kw)
    torch.cuda.synchronize()
    assert rel_l2(host(fused), host(chain).astype(np.float64)) <= 1e-3
    pos = host(pos0)[:, None, None] + np.arange(Tq)[None, None, :]
    qo, ro = nr.norm_rope(host(q), host(gq), pos), nr.norm_rope(host(r), host(gr), pos)
    lens = x["seq_lens"].cpu().numpy()
    for b in range(B):  # row t of sequence b sees the keys before position L_b - (Tq - 1 - t): causal over its own length
        ref = oracle.forward(qo[b:b + 1], ro[b:b + 1], host(x["k"])[b:b + 1, :, :lens[b]], host(x["v"])[b:b + 1, :, :lens[b]],
                             x["scale"], causal=True)
        got = host(fused)[b:b + 1].reshape(1, Hq, Tq, d)
        assert rel_l2(got, ref) <= BF16_REL_L2, b


def test_preparation_arguments_are_validated(plx):
    from paper_2605_29157_amd import synth

    y = synth.prefill_inputs(1, 4, 2, 64, 128, seed=60, device=DEV)
    g = torch.ones(128, dtype=torch.float32, device=DEV)
    table = plx.parallax_rope_table(64, 128, device=DEV)
    with pytest.raises(plx.ParallaxError):   # rotation asked for, no table
        bad = plx.qr_prep(g, g, None, None)
        bad.rope_q = 1
        plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], prep=bad)
    with pytest.raises(plx.ParallaxError):   # not together with a window
        plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], prep=plx.qr_prep(g, g, table), window=16)
    with pytest.raises(plx.ParallaxError):   # not together with the row cache
        plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], prep=plx.qr_prep(g, g, table),
                             save_for_backward=True)
    with pytest.raises(plx.ParallaxError):
        plx.parallax_rope_table(16, 127, device=DEV)
    with pytest.raises(plx.ParallaxError):   # weights must be 16-byte aligned (fetched four at a time)
        g2 = torch.ones(132, dtype=torch.float32, device=DEV)[1:129]
        bad = plx.qr_prep(g, g, table)
        bad.q_gamma = g2.data_ptr()
        plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], prep=bad)


def test_prefill_preparing_q_and_rho_at_the_benchmark_launch(plx, nr, oracle):
    """The launch bench.py times for the in-kernel preparation (config-4 shape, theta 1e6,
    positions 0..4095): oracle chain on a row of every workgroup plus the first and last 128 rows
    of two heads -- norm + rope in float64 on the raw rows, then the attention oracle on the
    prepared keys."""
    from paper_2605_29157_amd import synth

    B, T, Hq, Hkv, d = 4, 4096, 16, 8, 128
    y = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=1009, device=DEV, k_offset_sigma=0.5)
    gq, gr, gk = (1.0 + 0.1 * _rand((d,), 71 + i, torch.float32) for i in range(3))
    (k2,) = plx.parallax_norm_rope([(y["k"], gk, True)])
    table = plx.parallax_rope_table(T, d, device=DEV)
    out = plx.parallax_prefill(y["q"], y["r"], k2, y["v"], y["scale"], causal=True,
                               prep=plx.qr_prep(gq, gr, table, None))
    torch.cuda.synchronize()
    got = host(out)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(72)
    rows = {(b, h, int(rng.integers(blk, blk + 128))) for b in range(B) for h in range(Hq) for blk in range(0, T, 128)}
    for (b, h) in ((0, 0), (3, 15)):
        rows |= {(b, h, i) for i in list(range(128)) + list(range(T - 128, T))}
    rows = np.array(sorted(rows), dtype=np.int32)
    # the sampled rows, prepared by the oracle (one row block per sampled row: [1, 1, 1, d])
    qs = host(y["q"])[rows[:, 0], rows[:, 1], rows[:, 2]][:, None, None, :]
    rs = host(y["r"])[rows[:, 0], rows[:, 1], rows[:, 2]][:, None, None, :]
    pos = rows[:, 2][:, None, None]
    qo, ro = nr.norm_rope(qs, host(gq), pos)[:, 0, 0], nr.norm_rope(rs, host(gr), pos)[:, 0, 0]
    ko = nr.norm_rope(host(y["k"]), host(gk), np.arange(T)[None, None, :])
    # attention oracle row by row through its row-sample interface: put the prepared rows back
    # into otherwise-zero q, r tensors (only the sampled rows are evaluated)
    qfull, rfull = np.zeros((B, Hq, T, d)), np.zeros((B, Hq, T, d))
    qfull[rows[:, 0], rows[:, 1], rows[:, 2]] = qo
    rfull[rows[:, 0], rows[:, 1], rows[:, 2]] = ro
    ref = oracle.forward(qfull, rfull, ko, host(y["v"]), y["scale"], causal=True, rows=rows)
    sub = got[rows[:, 0], rows[:, 1], rows[:, 2]]
    assert rel_l2(sub, ref) <= BF16_REL_L2
    per_row = np.linalg.norm(sub - ref, axis=1) / np.linalg.norm(ref, axis=1)
    assert per_row.max() <= 5e-2, rows[int(per_row.argmax())]


def test_norm_rope_from_the_table_matches_the_in_kernel_evaluation(plx, nr):
    """(cos, sin) from parallax_rope_table instead of the kernel's own evaluation: a decode step's
    rows (T = 1 at positions up to 130 000) and a prefill chunk, bf16 and fp32, against the oracle
    and against the evaluating kernel."""
    for (B, H, T, d, dtype, p0) in [(4, 16, 1, 128, torch.bfloat16, [0, 77, 4095, 129999]),
                                    (2, 6, 70, 64, torch.bfloat16, [5, 1000]),
                                    (2, 4, 9, 32, torch.float32, [0, 300])]:
        x = _rand((B, H, T, d), 900 + T, dtype)
        gam = 1.0 + 0.2 * _rand((d,), 901, torch.float32)
        pos0 = torch.tensor(p0, dtype=torch.int32, device=DEV)
        table = plx.parallax_rope_table(max(p0) + T, d, device=DEV)
        (a,) = plx.parallax_norm_rope([(x, gam, True)], pos0=pos0, rope_table=table)
        (b,) = plx.parallax_norm_rope([(x, gam, True)], pos0=pos0)
        torch.cuda.synchronize()
        pos = host(pos0)[:, None, None] + np.arange(T)[None, None, :]
        ref = nr.norm_rope(host(x), host(gam), pos)
        tol = BF16_REL_L2 if dtype == torch.bfloat16 else 1e-5
        assert rel_l2(host(a), ref) <= tol
        assert rel_l2(host(a), host(b).astype(np.float64)) <= (2e-3 if dtype == torch.bfloat16 else 1e-5)
    # a table that is too short is clamped, never read past; a misaligned one is refused
    import ctypes
    x = _rand((1, 2, 4, 128), 910, torch.bfloat16)
    g = torch.ones(128, dtype=torch.float32, device=DEV)
    table = plx.parallax_rope_table(2, 128, device=DEV)
    plx.parallax_norm_rope([(x, g, True)], rope_table=table)
    a = plx.norm_rope_args([(x, g, True, torch.empty_like(x))], rope_table=table)
    a.rope_table += 4
    st = plx.load_library().parallax_norm_rope(ctypes.byref(a), int(torch.cuda.current_stream().cuda_stream))
    assert st == plx.PLX_ERR_ALIGN
    torch.cuda.synchronize()
