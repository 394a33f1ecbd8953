"""GPU tests of parallax_decode_fused: the merge done by the last split to arrive, inside the
split kernel. Same records, same merge order as the two-kernel path, so the outputs must be
bit-identical to parallax_decode's for the same split count; the oracle check rides along."""
import numpy as np
import pytest
import torch

from parity import BF16_REL_L2, host, oracle_decode, rel_l2

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
def counters():
    """One counter array shared by every call of this module: cleared once, then every call
    must leave it all zero (checked after each use)."""
    return torch.zeros(4096, dtype=torch.int32, device=DEV)


def _both(plx, x, counters, **kw):
    args = (x["q"], x["r"], x["k"], x["v"], x["scale"])
    two = plx.parallax_decode(*args, seq_lens=x.get("seq_lens"), **kw)
    one = plx.parallax_decode_fused(*args, counters, seq_lens=x.get("seq_lens"), **kw)
    torch.cuda.synchronize()
    assert int(counters.abs().sum().item()) == 0, "counters not returned to zero"
    return host(one), host(two)


@pytest.mark.parametrize("B,Hq,Hkv,L,d,S", [
    (8, 16, 8, 4096, 128, 0),     # benchmark configuration 2, library heuristic
    (3, 8, 4, 1500, 128, 5),      # ragged tail, odd split count
    (3, 8, 4, 1500, 128, 128),    # most splits empty
    (2, 8, 1, 777, 128, 3),       # one kv head, group of 8
    (2, 16, 1, 777, 128, 3),      # group of 16: every MFMA column is a head
    (2, 8, 4, 700, 64, 4),        # d = 64
    (1, 2, 2, 300, 128, 2),
    (2, 4, 2, 64, 128, 1),        # one split: no records, no counters touched
])
def test_fused_equals_two_kernels_bitwise(plx, synth, oracle, counters, B, Hq, Hkv, L, d, S):
    x = synth.decode_inputs(B, Hq, Hkv, L, d, seed=7000 + L + S, device=DEV, ragged=B > 1)
    one, two = _both(plx, x, counters, num_splits=S)
    np.testing.assert_array_equal(one, two)
    assert rel_l2(one, oracle_decode(oracle, x)) <= BF16_REL_L2


def test_fused_zero_length_sequence_and_twin(plx, synth, oracle, counters):
    x = synth.decode_inputs(4, 16, 8, 900, 128, seed=7101, device=DEV)
    x["seq_lens"] = torch.tensor([900, 0, 1, 513], dtype=torch.int32, device=DEV)
    one, two = _both(plx, x, counters, num_splits=6)
    np.testing.assert_array_equal(one, two)
    assert (one[1] == 0).all()
    one0, two0 = _both(plx, x, counters, num_splits=6, use_r=False)
    np.testing.assert_array_equal(one0, two0)
    assert rel_l2(one0, oracle_decode(oracle, x, use_r=False)) <= BF16_REL_L2


def test_fused_paged_cache_and_several_query_rows(plx, synth, counters):
    x = synth.decode_inputs(3, 16, 8, 1500, 128, seed=7102, device=DEV, ragged=True)
    kp, vp, table = synth.paged_cache(x, 48, seed=7103)
    kw = dict(seq_lens=x["seq_lens"], num_splits=4, block_table=table, max_len=1500)
    two = plx.parallax_decode(x["q"], x["r"], kp, vp, x["scale"], **kw)
    one = plx.parallax_decode_fused(x["q"], x["r"], kp, vp, x["scale"], counters, **kw)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(one), host(two))
    # Tq = 5 rows x group of 2: ten merged rows per (batch, kv head) group
    more = synth.prefill_inputs(3, 16, 8, 5, 128, seed=7104, device=DEV)
    q4, r4 = more["q"].contiguous(), more["r"].contiguous()
    two = plx.parallax_decode(q4, r4, x["k"], x["v"], x["scale"], seq_lens=x["seq_lens"], num_splits=5)
    one = plx.parallax_decode_fused(q4, r4, x["k"], x["v"], x["scale"], counters,
                                    seq_lens=x["seq_lens"], num_splits=5)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(one), host(two))
    assert int(counters.abs().sum().item()) == 0


def test_fused_repeated_calls_and_changing_shapes_share_counters(plx, synth, counters):
    """Back-to-back launches on one stream with no host synchronisation between them: each
    launch finds the counters its predecessor put back to zero."""
    shapes = [(8, 16, 8, 4096, 0), (2, 8, 4, 1000, 7), (16, 16, 8, 2048, 2), (8, 16, 8, 4096, 0)]
    xs = [synth.decode_inputs(B, Hq, Hkv, L, 128, seed=7200 + i, device=DEV)
          for i, (B, Hq, Hkv, L, _) in enumerate(shapes)]
    refs = [plx.parallax_decode(x["q"], x["r"], x["k"], x["v"], x["scale"], num_splits=s[4])
            for x, s in zip(xs, shapes)]
    ws = torch.empty(16 * 16 * 128 * (2 * 128 + 4), dtype=torch.float32, device=DEV)
    torch.cuda.synchronize()
    outs = []
    for rep in range(3):
        for x, s in zip(xs, shapes):
            outs.append(plx.parallax_decode_fused(x["q"], x["r"], x["k"], x["v"], x["scale"], counters,
                                                  num_splits=s[4], workspace=ws))
    torch.cuda.synchronize()
    for i, o in enumerate(outs):
        np.testing.assert_array_equal(host(o), host(refs[i % len(shapes)]))
    assert int(counters.abs().sum().item()) == 0


def test_fused_rejects_missing_or_short_counters(plx, synth):
    x = synth.decode_inputs(2, 4, 2, 600, 128, seed=7300, device=DEV)
    with pytest.raises(TypeError):
        plx.parallax_decode_fused(x["q"], x["r"], x["k"], x["v"], x["scale"],
                                  torch.zeros(3, dtype=torch.int32, device=DEV), num_splits=2)
    xf = synth.decode_inputs(2, 4, 2, 64, 64, seed=7301, dtype=torch.float32, device=DEV)
    with pytest.raises(plx.ParallaxError):
        plx.parallax_decode_fused(xf["q"], xf["r"], xf["k"], xf["v"], xf["scale"],
                                  torch.zeros(8, dtype=torch.int32, device=DEV))
