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
