"""parallax_decode_static (the decode entry point that allocates nothing: split records in a
fixed array inside the library) against parallax_decode with a caller-owned workspace, through
the C ABI: same kernels, same split count, so the outputs must agree bit for bit -- and, like
every decode result, with the CPU oracle to the bf16 bound."""
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


def _both(plx, x, **kw):
    """(static-scratch output, workspace output); the static call runs between two synchronisations
    with torch's allocator watched: it must not take device memory from it either."""
    want = plx.parallax_decode(x["q"], x["r"], x["k"], x["v"], x["scale"], seq_lens=x.get("seq_lens"), **kw)
    out = torch.full_like(x["q"], float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated(), torch.cuda.memory_reserved()
    plx.parallax_decode_static(x["q"], x["r"], x["k"], x["v"], x["scale"], out,
                               seq_lens=x.get("seq_lens"), **kw)
    torch.cuda.synchronize()
    assert (torch.cuda.memory_allocated(), torch.cuda.memory_reserved()) == before
    return host(out), host(want)


def test_two_calls_in_a_row_second_one_smaller(plx, synth, oracle):
    # first call: config-2 shape with the heuristic's split count (8 splits, 1 MB of records)
    big = synth.decode_inputs(8, 16, 8, 4096, 128, seed=2101, device=DEV, ragged=True)
    assert plx.parallax_decode_num_splits(8, 16, 8, 4096, 128) > 1
    got, want = _both(plx, big)
    np.testing.assert_array_equal(got, want)
    assert rel_l2(got, oracle_decode(oracle, big)) <= BF16_REL_L2
    # second call, smaller in every dimension, over the first call's stale records
    small = synth.decode_inputs(2, 4, 2, 1500, 128, seed=2102, device=DEV, ragged=True)
    for S in (0, 5):
        got, want = _both(plx, small, num_splits=S)
        np.testing.assert_array_equal(got, want)
        assert rel_l2(got, oracle_decode(oracle, small)) <= BF16_REL_L2
    # and the first one again
    got, want = _both(plx, big)
    np.testing.assert_array_equal(got, want)


def test_variants_share_the_scratch(plx, synth, oracle):
    # d = 64, many splits with empty ones, a zero-length sequence
    x = synth.decode_inputs(3, 8, 4, 777, 64, seed=2103, device=DEV, ragged=True)
    x["seq_lens"][1] = 0
    for S in (1, 4, 128):
        got, want = _both(plx, x, num_splits=S)
        np.testing.assert_array_equal(got, want)
        assert np.all(got[1] == 0.0)
    # several query rows per sequence, sliding window, softmax-only twin
    y = synth.decode_inputs(2, 4, 2, 1200, 128, seed=2104, device=DEV)
    gen = torch.Generator(DEV).manual_seed(9)
    y["q"] = torch.randn(2, 4, 3, 128, device=DEV, generator=gen).to(torch.bfloat16)
    y["r"] = torch.randn(2, 4, 3, 128, device=DEV, generator=gen).to(torch.bfloat16)
    for kw in (dict(num_splits=3), dict(num_splits=4, window=300), dict(num_splits=2, use_r=False)):
        got, want = _both(plx, y, **kw)
        np.testing.assert_array_equal(got, want)


def test_records_beyond_the_scratch_are_refused(plx, synth):
    assert plx.parallax_decode_static_scratch_bytes() == plx.PLX_STATIC_SCRATCH_RECORDS * (2 * 128 + 4) * 4
    # 17 sequences x 8 heads x 128 splits = 17 408 records of d = 128: more than 16 384
    x = synth.decode_inputs(17, 8, 8, 256, 128, seed=2105, device=DEV)
    out = torch.zeros_like(x["q"])
    with pytest.raises(plx.ParallaxError) as e:
        plx.parallax_decode_static(x["q"], x["r"], x["k"], x["v"], x["scale"], out, num_splits=128)
    assert e.value.status == plx.PLX_ERR_SCRATCH
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0  # nothing was enqueued
    # 16 sequences are exactly the limit; at d = 64 twice as many records fit
    x16 = {n: (t[:16] if torch.is_tensor(t) else t) for n, t in x.items()}
    got, want = _both(plx, x16, num_splits=128)
    np.testing.assert_array_equal(got, want)
