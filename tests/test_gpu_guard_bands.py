"""Out-of-bounds canaries: every buffer an entry point WRITES (outputs, split workspace, row cache,
gradients) sits inside a larger allocation filled with a sentinel byte; after the call the bands
in front of and behind it must be untouched. Shapes with ragged tails (lengths that are not
multiples of the tiles) are where a stray store would land. Every kernel runs on valid arguments
and exits normally; the check itself is on the host."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GUARD = 64 * 1024  # bytes on each side
SENTINEL = 0xA5


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


class Guarded:
    """Tensors carved out of sentinel-filled allocations."""

    def __init__(self):
        self.blocks = []

    def empty(self, shape, dtype):
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        raw = torch.full((GUARD + n + GUARD,), SENTINEL, dtype=torch.uint8, device=DEV)
        assert raw.data_ptr() % 256 == 0
        view = raw[GUARD:GUARD + n].view(dtype).view(shape)
        self.blocks.append((raw, n, tuple(shape)))
        return view

    def like(self, t):
        return self.empty(tuple(t.shape), t.dtype)

    def check(self, what):
        torch.cuda.synchronize()
        for raw, n, shape in self.blocks:
            front, back = raw[:GUARD], raw[GUARD + n:]
            assert bool((front == SENTINEL).all()), (what, shape, "store in front of the buffer")
            assert bool((back == SENTINEL).all()), (what, shape, "store behind the buffer")


def _call(plx, entry, args):
    st = getattr(plx.load_library(), entry)(ctypes.byref(args), int(torch.cuda.current_stream().cuda_stream))
    assert st == 0, (entry, plx.strerror(st))


@pytest.mark.parametrize("B,Hq,Hkv,L,d,S,Tq", [(3, 8, 4, 777, 128, 5, 1), (2, 4, 2, 1500, 64, 128, 1),
                                                (2, 4, 2, 1001, 128, 3, 3), (1, 8, 1, 300, 128, 4, 5),
                                                (2, 16, 8, 130, 128, 1, 1)])
def test_decode_outputs_and_workspace(plx, synth, B, Hq, Hkv, L, d, S, Tq):
    x = synth.decode_inputs(B, Hq, Hkv, L, d, seed=7100 + L, device=DEV, ragged=True)
    if Tq > 1:
        gen = torch.Generator(DEV).manual_seed(7)
        x["q"] = torch.randn(B, Hq, Tq, d, device=DEV, generator=gen).to(torch.bfloat16)
        x["r"] = torch.randn(B, Hq, Tq, d, device=DEV, generator=gen).to(torch.bfloat16)
    for entry in ("parallax_decode", "parallax_decode_fused", "parallax_decode_partials"):
        g = Guarded()
        out = g.like(x["q"])
        # exactly the bytes the call needs: a record too many would land in the band
        ws = g.empty((B * Hq * Tq * S * (2 * d + 4),), torch.float32) if (S > 1 or "partials" in entry) else None
        a = plx.decode_args(x["q"], x["r"], x["k"], x["v"], out, x["scale"], x["seq_lens"], True, S, ws)
        if entry == "parallax_decode_fused":
            counters = g.empty((B * Hkv,), torch.int32)
            counters.zero_()
            a.split_counters = counters.data_ptr()
        _call(plx, entry, a)
        g.check((entry, B, Hq, Hkv, L, d, S, Tq))
    if S > 1:  # and the merge on its own
        g = Guarded()
        out = g.like(x["q"])
        ws = torch.zeros(B * Hq * Tq * S * (2 * d + 4), dtype=torch.float32, device=DEV)
        a = plx.decode_args(x["q"], x["r"], x["k"], x["v"], out, x["scale"], x["seq_lens"], True, S, ws)
        _call(plx, "parallax_decode_combine", a)
        g.check(("parallax_decode_combine", B, Hq, L, d, S, Tq))


def test_decode_paged_window_and_static(plx, synth):
    x = synth.decode_inputs(3, 8, 4, 900, 128, seed=7200, device=DEV, ragged=True)
    kp, vp, table = synth.paged_cache(x, 48, seed=7201)
    for kw in (dict(block_table=table, max_len=900), dict(window=200)):
        g = Guarded()
        out = g.like(x["q"])
        ws = g.empty((3 * 8 * 4 * (2 * 128 + 4),), torch.float32)
        k, v = (kp, vp) if "block_table" in kw else (x["k"], x["v"])
        a = plx.decode_args(x["q"], x["r"], k, v, out, x["scale"], x["seq_lens"], True, 4, ws, **kw)
        _call(plx, "parallax_decode", a)
        g.check(("parallax_decode", kw.keys()))
    g = Guarded()
    out = g.like(x["q"])
    a = plx.decode_args(x["q"], x["r"], x["k"], x["v"], out, x["scale"], x["seq_lens"], True, 6, None)
    _call(plx, "parallax_decode_static", a)
    g.check("parallax_decode_static")


@pytest.mark.parametrize("B,Hq,L,S", [(3, 16, 700, 4), (2, 20, 130, 1), (1, 40, 1000, 7)])
def test_decode_mla_outputs_and_workspace(plx, synth, B, Hq, L, S):
    x = synth.mla_decode_inputs(B, Hq, L, seed=7300 + L, device=DEV, ragged=True)
    g = Guarded()
    out = g.empty((B, Hq, 512), torch.bfloat16)
    ws = g.empty((B * Hq * S * (2 * 512 + 4),), torch.float32) if S > 1 else None
    a = plx.decode_mla_args(x["q"], x["r"], x["ckv"], out, x["scale"], x["seq_lens"], S, ws)
    _call(plx, "parallax_decode_mla", a)
    g.check(("parallax_decode_mla", B, Hq, L, S))


@pytest.mark.parametrize("Hq,Tq,L,S,W", [(5, 3, 700, 4, 0), (2, 70, 130, 1, 0), (16, 2, 1000, 7, 200)])
def test_decode_mla_rows_and_window(plx, synth, Hq, Tq, L, S, W):
    B = 2
    x = synth.mla_decode_inputs(B, Hq * Tq, L, seed=7350 + L, device=DEV, ragged=True)
    q, r = x["q"].view(B, Hq, Tq, 576), x["r"].view(B, Hq, Tq, 576)
    g = Guarded()
    out = g.empty((B, Hq, Tq, 512), torch.bfloat16)
    ws = g.empty((B * Hq * Tq * S * (2 * 512 + 4),), torch.float32) if S > 1 else None
    a = plx.decode_mla_args(q, r, x["ckv"], out, x["scale"], x["seq_lens"], S, ws, window=W)
    _call(plx, "parallax_decode_mla", a)
    g.check(("parallax_decode_mla", Hq, Tq, L, S, W))


@pytest.mark.parametrize("T,Tkv,d,causal,window", [(300, 300, 128, True, 0), (129, 129, 64, True, 0),
                                                    (77, 500, 128, True, 0), (300, 300, 128, False, 0),
                                                    (333, 333, 128, True, 50), (1, 1, 128, True, 0),
                                                    (200, 333, 64, True, 100)])
def test_prefill_output_row_cache_and_gradients(plx, synth, T, Tkv, d, causal, window):
    B, Hq, Hkv = 2, 4, 2
    y = synth.prefill_inputs(B, Hq, Hkv, Tkv, d, seed=7400 + T, device=DEV)
    q, r = y["q"][:, :, Tkv - T:].contiguous(), y["r"][:, :, Tkv - T:].contiguous()
    # forward alone
    g = Guarded()
    out = g.like(q)
    a = plx.prefill_args(q, r, y["k"], y["v"], out, y["scale"], causal, True, window)
    _call(plx, "parallax_prefill", a)
    g.check(("parallax_prefill", T, Tkv, d, causal, window))
    # forward with the row cache
    g = Guarded()
    out, vbar = g.like(q), g.like(q)
    stats = g.empty((B, Hq, T, 2), torch.float32)
    a = plx.prefill_args(q, r, y["k"], y["v"], out, y["scale"], causal, True, window)
    a.vbar, a.row_stats = vbar.data_ptr(), stats.data_ptr()
    _call(plx, "parallax_prefill", a)
    g.check(("parallax_prefill + row cache", T, Tkv, d, causal, window))
    # backward: gradients and the row-scalar workspace
    g2 = Guarded()
    dq, dr, dk, dv = g2.like(q), g2.like(q), g2.like(y["k"]), g2.like(y["k"])
    ws = g2.empty((B * Hq * T * 4,), torch.float32)
    d_o = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=7401, device=DEV)["q"].contiguous()
    a = plx.prefill_bwd_args(q, r, y["k"], y["v"], out, vbar, stats, d_o, dq, dr, dk, dv, y["scale"], causal,
                             ws, window)
    _call(plx, "parallax_prefill_backward", a)
    g2.check(("parallax_prefill_backward", T, Tkv, d, causal, window))
    g.check(("parallax_prefill_backward reads", T, Tkv, d, causal, window))


def test_prefill_fp32_block_sparse_and_norm_rope(plx, synth):
    # fp32 forward + backward
    y = synth.prefill_inputs(1, 2, 2, 70, 64, seed=7500, dtype=torch.float32, device=DEV)
    g = Guarded()
    out, vbar = g.like(y["q"]), g.like(y["q"])
    stats = g.empty((1, 2, 70, 2), torch.float32)
    a = plx.prefill_args(y["q"], y["r"], y["k"], y["v"], out, y["scale"], True, True, 0)
    a.vbar, a.row_stats = vbar.data_ptr(), stats.data_ptr()
    _call(plx, "parallax_prefill", a)
    dq, dr, dk, dv = g.like(y["q"]), g.like(y["q"]), g.like(y["k"]), g.like(y["k"])
    ws = g.empty((1 * 2 * 70 * 4,), torch.float32)
    a = plx.prefill_bwd_args(y["q"], y["r"], y["k"], y["v"], out, vbar, stats, y["v"].clone(), dq, dr, dk, dv,
                             y["scale"], True, ws, 0)
    _call(plx, "parallax_prefill_backward", a)
    g.check("fp32 prefill + backward")
    # block-sparse forward with empty row blocks and a ragged last tile
    y = synth.prefill_inputs(2, 4, 2, 450, 128, seed=7501, device=DEV)
    bm = torch.as_tensor(np.random.default_rng(7502).random((4, 8)) < 0.4, device=DEV)
    bm[2] = False
    g = Guarded()
    out = g.like(y["q"])
    row_ptr, tile_idx, Bs, Hs = plx.block_mask_lists(bm)
    a = plx.prefill_args(y["q"], y["r"], y["k"], y["v"], out, y["scale"], True, True)
    a.sparse_row_ptr, a.sparse_tile_idx, a.sparse_batch, a.sparse_heads = row_ptr.data_ptr(), tile_idx.data_ptr(), Bs, Hs
    _call(plx, "parallax_prefill", a)
    g.check("block-sparse prefill")
    # ... with the row cache, and the backward over the same lists (row and column form)
    g = Guarded()
    out, vbar = g.like(y["q"]), g.like(y["q"])
    stats = g.empty((2, 4, 450, 2), torch.float32)
    a.o, a.vbar, a.row_stats = out.data_ptr(), vbar.data_ptr(), stats.data_ptr()
    _call(plx, "parallax_prefill", a)
    g.check("block-sparse prefill + row cache")
    g2 = Guarded()
    dq, dr, dk, dv = g2.like(y["q"]), g2.like(y["q"]), g2.like(y["k"]), g2.like(y["k"])
    ws = g2.empty((2 * 4 * 450 * 4,), torch.float32)
    ba = plx.prefill_bwd_args(y["q"], y["r"], y["k"], y["v"], out, vbar, stats, y["q"], dq, dr, dk, dv, y["scale"],
                              True, ws)
    col_ptr, col_idx = plx.block_mask_column_lists(bm)
    ba.sparse_row_ptr, ba.sparse_tile_idx = row_ptr.data_ptr(), tile_idx.data_ptr()
    ba.sparse_col_ptr, ba.sparse_col_idx = col_ptr.data_ptr(), col_idx.data_ptr()
    ba.sparse_batch, ba.sparse_heads = Bs, Hs
    _call(plx, "parallax_prefill_backward", ba)
    g2.check("block-sparse backward")
    g.check("block-sparse backward reads")
    # RMSNorm + RoPE out of place
    g = Guarded()
    gam = torch.ones(128, dtype=torch.float32, device=DEV)
    outs = [g.like(y[n]) for n in ("q", "r", "k")]
    a = plx.norm_rope_args([(y["q"], gam, True, outs[0]), (y["r"], gam, True, outs[1]), (y["k"], gam, False, outs[2])])
    _call(plx, "parallax_norm_rope", a)
    g.check("parallax_norm_rope")
