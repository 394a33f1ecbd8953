#!/usr/bin/env python3
"""Benchmark of the Parallax attention hot path on one MI355X.

Default workload (benchmark configuration 2): single-step decode, bf16, B=8, 16 query heads / 8 KV
heads (GQA group 2), head_dim 128, KV context 4096. One "step" = one parallax_decode call:
the split-KV kernel over the whole KV cache plus the combine kernel. Inputs are synthetic
(seeded N(0,1)), resident in HBM before the timed region; 8 distinct KV caches (1.07 GB) are
rotated so that no step finds its cache in the 256 MB Infinity Cache.

Prints ONE JSON line. `value` is algorithmic KV bytes per second over the timed steps;
`roofline` times the dominant kernel (the split-KV kernel alone, via
parallax_decode_partials) with events on the launch stream; `cpu_baseline` times the
double-precision CPU oracle on the same batch; `extra` carries the decode sweep, the
softmax-only twin and the causal prefill TFLOP/s.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0       # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0
PREROLL_SECONDS = 0.06  # untimed load in front of every timed loop (see _preroll)

# HBM bytes per launch of the dominant kernels, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled
# by the same counters on parallax_util_copy of known size: written by
# `python3 -m paper_2605_29157_amd.profiling traffic ... --out profiles/hbm_traffic.txt` from the
# counter runs described in profiles/*_hbm_counters.md; a key that is not there reads as null.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")


def measured_traffic(key):
    from paper_2605_29157_amd.profiling import read_traffic_file

    return read_traffic_file(TRAFFIC_FILE).get(key)


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def decode_bytes(B, Hkv, d, lens_sum, Hq):
    """Algorithmic bytes of one decode step: K and V once, q, r read and o written (bf16)."""
    return Hkv * lens_sum * d * 2 * 2 + B * Hq * d * 2 * 3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--no-extra", action="store_true", help="skip the sweep / prefill lines")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--workload", choices=["decode", "prefill", "backward", "sweep", "mla"], default="decode",
                    help="decode = config 2 (the headline line); prefill = config 4 causal "
                         "prefill alone, for profiling that kernel; backward = the backward pass "
                         "of that prefill shape; sweep = the config 3 decode "
                         "grid (B x L, fixed and ragged lengths, d = 128 and 64), one JSON line; "
                         "mla = attention over a latent cache alone (--mla-shape)")
    ap.add_argument("--mla-shape", default="16,128,1,8192", metavar="B,Hq,Tq,L",
                    help="sequences, heads, rows per head and cached tokens of the latent-cache workload "
                         "(default: 128 heads on one GPU; up to 16 heads x rows run the memory-bound "
                         "kernel, more the 32-column one)")
    ap.add_argument("--decode-shape", default="8,4096", metavar="B,L",
                    help="batch and KV length of the decode workload (default 8,4096 = config 2; "
                         "other shapes are for profiling the same kernels at larger sizes)")
    ap.add_argument("--prefill-shape", default="4,4096", metavar="B,T",
                    help="batch and length of the causal prefill workload (default 4,4096 = config 4)")
    ap.add_argument("--prefill-heads", default="16,8,128", metavar="Hq,Hkv,d",
                    help="query heads, KV heads and head dimension of the prefill workload "
                         "(default 16,8,128; 32,16,64 is the compute-matched layout)")
    ap.add_argument("--counter-mode", action="store_true",
                    help="short run for hardware-counter collection: 5 launches of the plain copy "
                         "kernel on 1 GiB (known size, calibrates FETCH_SIZE / WRITE_SIZE) and "
                         "--steps launches of the split-KV kernel (with --workload prefill: of the "
                        "prefill kernel); prints nothing to parse")
    opt = ap.parse_args()
    if opt.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path "
              "(--gpus %d refused; run with --gpus 1)" % opt.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2605_29157_amd import binding as plx
    from paper_2605_29157_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    lib = plx.load_library()
    stream = torch.cuda.current_stream()
    sptr = int(stream.cuda_stream)

    if opt.workload == "prefill":
        print(json.dumps(prefill_line(torch, plx, synth, dev, opt)))
        return
    if opt.workload == "backward":
        print(json.dumps(backward_line(torch, plx, synth, dev, opt)))
        return
    if opt.workload == "sweep":
        print(json.dumps(decode_sweep(torch, plx, synth, lib, dev, sptr)))
        return
    if opt.workload == "mla":
        print(json.dumps(mla_line(torch, plx, synth, lib, dev, sptr, opt)))
        return

    # ------------------------------------------------------------------ workload: config 2
    B, L = (int(v) for v in opt.decode_shape.split(","))
    Hq, Hkv, d = 16, 8, 128
    is_config2 = (B, L) == (8, 4096)
    # rotate enough KV caches that no step finds its cache in the 256 MB Infinity Cache
    NSETS = max(2, min(8, int(2.2e9 // (B * Hkv * L * d * 4))))
    sets = [synth.decode_inputs(B, Hq, Hkv, L, d, seed=1002 + 10 * i, device=dev) for i in range(NSETS)]
    S = plx.parallax_decode_num_splits(B, Hq, Hkv, L, d)
    ws = torch.empty(plx.parallax_decode_workspace_bytes(B, Hq, Hkv, L, d) // 4,
                     dtype=torch.float32, device=dev)
    out = torch.empty_like(sets[0]["q"])
    full_args = [plx.decode_args(x["q"], x["r"], x["k"], x["v"], out, x["scale"], None, True, 0, ws)
                 for x in sets]
    part_args = [plx.decode_args(x["q"], x["r"], x["k"], x["v"], out, x["scale"], None, True, S, ws)
                 for x in sets]
    step_bytes = decode_bytes(B, Hkv, d, B * L, Hq)

    def run(fn, arglist, n):
        for i in range(n):
            st = fn(ctypes.byref(arglist[i % NSETS]), sptr)
            if st != 0:
                raise plx.ParallaxError(st, "bench step")

    if opt.counter_mode:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).zero_()
        dst = torch.empty_like(src)
        for _ in range(5):
            plx.parallax_util_copy(dst, src)
        run(lib.parallax_decode_partials, part_args, opt.steps)
        torch.cuda.synchronize()
        print(json.dumps({"counter_mode": True, "copy_bytes_each_way": src.numel(),
                          "decode_algorithmic_bytes": step_bytes, "num_splits": S}))
        return

    # ------------------------------------------------------------------ timed region
    _preroll(torch, lambda: run(lib.parallax_decode, full_args, NSETS))
    run(lib.parallax_decode, full_args, opt.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(lib.parallax_decode, full_args, opt.steps)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sec_per_step = (t1 - t0) / opt.steps
    value = step_bytes / sec_per_step / 1e9

    # same K steps between events on the launch stream (excludes host launch gaps at the ends)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    run(lib.parallax_decode, full_args, opt.steps)
    e1.record(stream)
    torch.cuda.synchronize()
    step_us_events = e0.elapsed_time(e1) * 1e3 / opt.steps

    # ------------------------------------------------------------------ roofline: split-KV kernel
    _preroll(torch, lambda: run(lib.parallax_decode_partials, part_args, NSETS))
    run(lib.parallax_decode_partials, part_args, opt.warmup)
    torch.cuda.synchronize()
    e0.record(stream)
    run(lib.parallax_decode_partials, part_args, opt.steps)
    e1.record(stream)
    torch.cuda.synchronize()
    kern_us = e0.elapsed_time(e1) * 1e3 / opt.steps
    achieved = step_bytes / (kern_us * 1e-6) / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                "traffic": measured_traffic("decode_bf16_config2") if is_config2 else None,
                "kernel": "decode_bf16_kernel<128,true,false,false>", "kernel_us": round(kern_us, 2),
                "algorithmic_bytes_per_launch": step_bytes}

    # per-launch spread: one event pair per step (whole step) and per split-KV kernel launch
    def per_launch(fn, arglist, n):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for i, (a, b) in enumerate(evs):
            a.record(stream)
            st = fn(ctypes.byref(arglist[i % NSETS]), sptr)
            b.record(stream)
            if st != 0:
                raise plx.ParallaxError(st, "bench step")
        torch.cuda.synchronize()
        us = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
        return {"median": round(us[len(us) // 2], 2), "min": round(us[0], 2), "n": n}

    n_single = min(opt.steps, 200)
    step_spread = per_launch(lib.parallax_decode, full_args, n_single)
    roofline["kernel_us_single_launches"] = per_launch(lib.parallax_decode_partials, part_args, n_single)

    result = {
        "metric": "decode_hbm_bandwidth", "value": round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": opt.steps, "warmup": opt.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 5), "us_per_step": round(sec_per_step * 1e6, 2),
        "us_per_step_stream_events": round(step_us_events, 2),
        "us_per_step_single_launches": step_spread,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%sdecode bf16 B=%d Hq=16 Hkv=8 d=128 L=%d, "
                               "%d rotated KV caches (cache-cold)"
                               % ("config2: " if is_config2 else "", B, L, NSETS),
                   "num_splits": S, "bytes_per_step": step_bytes},
        "roofline": roofline,
    }

    # ------------------------------------------------------------------ CPU oracle baseline
    if not opt.no_cpu_baseline and is_config2:
        from oracle import parallax_oracle

        parallax_oracle.build()
        x = sets[0]
        qh = x["q"].float().cpu().numpy()[:, :, None, :]
        rh = x["r"].float().cpu().numpy()[:, :, None, :]
        kh, vh = x["k"].float().cpu().numpy(), x["v"].float().cpu().numpy()

        def time_oracle(budget_s):
            reps, tot, ref = 0, 0.0, None
            while tot < budget_s and reps < 1000:
                c0 = time.perf_counter()
                ref = parallax_oracle.forward(qh, rh, kh, vh, x["scale"])
                tot += time.perf_counter() - c0
                reps += 1
            return reps, tot, ref

        n_threads = parallax_oracle.num_threads()
        reps, tot, ref = time_oracle(10.0)  # about 10 s of oracle work on all host threads
        got = plx.parallax_decode(x["q"], x["r"], x["k"], x["v"], x["scale"], workspace=ws)
        torch.cuda.synchronize()
        err = float(np.linalg.norm(got.float().cpu().numpy()[:, :, None, :] - ref) /
                    np.linalg.norm(ref))
        result["cpu_baseline"] = {
            "value": round(step_bytes / (tot / reps) / 1e9, 3), "unit": "GB/s",
            "cores": n_threads, "kind": "oracle", "cpu_model": cpu_model(),
            "sample": "the full config-2 batch (8 sequences x 4096 keys), %d passes of the "
                      "double-precision C oracle, %.3f s each" % (reps, tot / reps),
            "gpu_vs_oracle_rel_l2": err,
        }
        # ... and on one thread (the oracle is OpenMP code: its runtime's own switch, the oracle
        # itself is not touched)
        try:
            gomp = ctypes.CDLL("libgomp.so.1")
            gomp.omp_set_num_threads(1)
            reps1, tot1, _ = time_oracle(5.0)
            gomp.omp_set_num_threads(n_threads)
            result["cpu_baseline"]["single_thread"] = {
                "value": round(step_bytes / (tot1 / reps1) / 1e9, 3), "unit": "GB/s", "cores": 1,
                "sample": "the same batch, %d passes, %.3f s each" % (reps1, tot1 / reps1)}
        except OSError:
            pass

    # ------------------------------------------------------------------ extra lines
    if not opt.no_extra and is_config2:
        result["extra"] = extra_measurements(torch, plx, synth, lib, dev, sptr, sets, ws, out)

    print(json.dumps(result))


def mla_line(torch, plx, synth, lib, dev, sptr, opt):
    """Attention over an MLA-style latent cache on its own (R21): Tq rows per head at the end of L
    cached tokens. Algorithmic flops: 2 * (2 * 576 + 2 * 512) per (head, row, visible token);
    algorithmic bytes: the cache once + q, rho, o."""
    B, Hq, Tq, L = (int(v) for v in opt.mla_shape.split(","))
    n_cols = Hq * Tq
    nset = max(1, min(8, int(2e9 // (B * L * 1152))))  # rotated caches: every call reads cold data
    xs = [synth.mla_decode_inputs(B, n_cols, L, seed=1040 + i, device=dev) for i in range(nset)]
    out = torch.empty(B, Hq, Tq, 512, dtype=torch.bfloat16, device=dev)
    S = plx.parallax_decode_mla_num_splits(B, n_cols, L)
    ws = torch.empty(max(B * n_cols * S * 1028, 4), dtype=torch.float32, device=dev)
    args = [plx.decode_mla_args(x["q"].view(B, Hq, Tq, 576), x["r"].view(B, Hq, Tq, 576), x["ckv"], out, x["scale"],
                                None, S, ws) for x in xs]
    k = [0]

    def step():
        st = lib.parallax_decode_mla(ctypes.byref(args[k[0] % nset]), sptr)
        k[0] += 1
        if st != 0:
            raise plx.ParallaxError(st, "mla bench")

    steps, warm = min(opt.steps, 100), min(opt.warmup, 5)
    us = _time_events(torch, step, warm, steps)
    pairs = B * Hq * sum(max(L - Tq + t + 1, 0) for t in range(Tq))
    flops = 4352.0 * pairs
    nbytes = B * L * 1152 + B * n_cols * (2 * 576 * 2 + 512 * 2)
    wide = n_cols > 16
    tf, gbps = flops / us / 1e6, nbytes / us / 1e3
    roof = ({"bound": "mfma", "achieved": round(tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
             "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None, "kernel": "decode_mla_wide_kernel"}
            if wide else
            {"bound": "hbm", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
             "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": None, "kernel": "decode_mla_kernel"})
    roof["step_us_incl_combine"] = round(us, 1)
    return {
        "metric": "latent_cache_attention_bf16", "value": round(tf if wide else gbps, 1),
        "unit": "TFLOP/s" if wide else "GB/s", "n_gpus": 1, "steps": steps, "warmup": warm,
        "ms_per_step": round(us / 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "latent cache (512 + 64) bf16 B=%d Hq=%d rows=%d L=%d, %d splits" % (B, Hq, Tq, L, S),
                   "algorithmic_flops": flops, "algorithmic_bytes": nbytes},
        "roofline": roof,
    }


def prefill_line(torch, plx, synth, dev, opt):
    """Config 4 on its own: causal prefill bf16 B=4 T=4096 Hq=16 Hkv=8 d=128."""
    B, T = (int(v) for v in opt.prefill_shape.split(","))
    Hq, Hkv, d = (int(v) for v in opt.prefill_heads.split(","))
    is_config4 = (B, T, Hq, Hkv, d) == (4, 4096, 16, 8, 128)
    y = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=1004, device=dev, k_offset_sigma=0.5)
    out = torch.empty_like(y["q"])
    steps = min(opt.steps, 50)
    warm = min(opt.warmup, 5)

    def step():
        plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=True, out=out)

    if opt.counter_mode:  # hardware-counter collection: the copy of known size, then the kernel
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).zero_()
        dst = torch.empty_like(src)
        for _ in range(5):
            plx.parallax_util_copy(dst, src)
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        return {"counter_mode": True, "copy_bytes_each_way": src.numel()}

    us = _time_events(torch, step, warm, steps)
    flops = B * Hq * 8 * d * T * (T + 1) / 2
    tf = flops / us / 1e6
    return {
        "metric": "prefill_bf16_throughput", "value": round(tf, 1), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": steps, "warmup": warm, "ms_per_step": round(us / 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "%scausal prefill bf16 B=%d T=%d Hq=%d Hkv=%d d=%d, "
                               "K offset N(0,0.5^2)" % ("config4: " if is_config4 else "", B, T, Hq, Hkv, d),
                   "algorithmic_flops": flops},
        "roofline": {"bound": "mfma", "achieved": round(tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                     "traffic": measured_traffic("prefill_bf16_config4") if is_config4 else None,
                     "kernel": "prefill_bf16_kernel<%d,true,true,false,false,false>" % d,
                     "kernel_us": round(us, 1)},
    }


def backward_line(torch, plx, synth, dev, opt):
    """Backward pass of the causal prefill shape (default config 4): rows prepare + dQ/dR pass +
    dK/dV pass, from the row cache a forward call left behind. 22 d flops per allowed (row, key)
    pair: eleven contractions of 2 d flops (five in the row pass, six in the column pass)."""
    B, T = (int(v) for v in opt.prefill_shape.split(","))
    Hq, Hkv, d = (int(v) for v in opt.prefill_heads.split(","))
    y = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=1004, device=dev, k_offset_sigma=0.5)
    g = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=1014, device=dev)["q"].contiguous()
    o, vbar, stats = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=True,
                                          save_for_backward=True)
    dq, dr = torch.empty_like(y["q"]), torch.empty_like(y["q"])
    dk, dv = torch.empty_like(y["k"]), torch.empty_like(y["k"])
    ws = torch.empty(plx.parallax_prefill_backward_workspace_bytes(B, Hq, T) // 4,
                     dtype=torch.float32, device=dev)
    a = plx.prefill_bwd_args(y["q"], y["r"], y["k"], y["v"], o, vbar, stats, g, dq, dr, dk, dv,
                             y["scale"], True, ws)
    lib = plx.load_library()
    sptr = int(torch.cuda.current_stream().cuda_stream)
    steps = min(opt.steps, 20)
    warm = min(opt.warmup, 3)

    def step():
        st = lib.parallax_prefill_backward(ctypes.byref(a), sptr)
        if st != 0:
            raise plx.ParallaxError(st, "parallax_prefill_backward")

    us = _time_events(torch, step, warm, steps)
    fwd_us = _time_events(
        torch, lambda: plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=True,
                                            out=o), warm, steps)
    # the forward as a training step runs it: with the row cache (o, vbar, lse, ubar) written
    fa = plx.prefill_args(y["q"], y["r"], y["k"], y["v"], o, y["scale"], True, True, 0)
    fa.vbar, fa.row_stats = vbar.data_ptr(), stats.data_ptr()

    def fwd_cache_step():
        st = lib.parallax_prefill(ctypes.byref(fa), sptr)
        if st != 0:
            raise plx.ParallaxError(st, "parallax_prefill")

    fwd_cache_us = _time_events(torch, fwd_cache_step, warm, steps)
    flops = B * Hq * 22 * d * T * (T + 1) / 2
    tf = flops / us / 1e6
    train_tf = B * Hq * 30 * d * T * (T + 1) / 2 / (us + fwd_cache_us) / 1e6
    return {
        "metric": "prefill_backward_bf16_throughput", "value": round(tf, 1), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": steps, "warmup": warm, "ms_per_step": round(us / 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "backward of causal prefill bf16 B=%d T=%d Hq=%d Hkv=%d d=%d, "
                               "K offset N(0,0.5^2)" % (B, T, Hq, Hkv, d),
                   "algorithmic_flops": flops, "forward_ms": round(fwd_us / 1e3, 4),
                   "forward_with_row_cache_ms": round(fwd_cache_us / 1e3, 4),
                   "forward_with_row_cache_plus_backward_TFLOPs": round(train_tf, 1)},
        "roofline": {"bound": "mfma", "achieved": round(tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                     "kernel": "bwd_dq_dr_kernel<%d,true,false> + bwd_dk_dv_kernel<%d,true,false>" % (d, d),
                     "kernel_us": round(us, 1)},
    }


def decode_sweep(torch, plx, synth, lib, dev, sptr):
    """Config 3: B in {1, 16, 64, 128} x L in {1024, 4096, 16384, 65536}, bf16, 16 query / 8 KV
    heads at d = 128 and the compute-matched 32 / 16 heads at d = 64; fixed lengths and ragged
    lengths uniform on [L/2, L]. KV caches are rotated (>= 1 GB in total where one is smaller)."""
    rows = []
    for (Hq, Hkv, d) in [(16, 8, 128), (32, 16, 64)]:
        for B in (1, 16, 64, 128):
            for L in (1024, 4096, 16384, 65536):
                per_set = B * Hkv * L * d * 4
                nset = max(1, min(8, int(1.2e9 // per_set) + 1))
                for ragged in (False, True):
                    xs = [synth.decode_inputs(B, Hq, Hkv, L, d, seed=3000 + i, device=dev,
                                              ragged=ragged) for i in range(nset)]
                    o = torch.empty_like(xs[0]["q"])
                    w = torch.empty(plx.parallax_decode_workspace_bytes(B, Hq, Hkv, L, d) // 4,
                                    dtype=torch.float32, device=dev)
                    row = {"d": d, "B": B, "L": L, "ragged": ragged, "kv_sets": nset,
                           "num_splits": plx.parallax_decode_num_splits(B, Hq, Hkv, L, d)}
                    lens_sum = [int(x["seq_lens"].sum().item()) if ragged else B * L for x in xs]
                    for use_r in (True, False):
                        al = [plx.decode_args(x["q"], x["r"], x["k"], x["v"], o, x["scale"],
                                              x.get("seq_lens"), use_r, 0, w) for x in xs]
                        c = [0]

                        def step():
                            lib.parallax_decode(ctypes.byref(al[c[0] % nset]), sptr)
                            c[0] += 1

                        iters = 200 if per_set < 2e8 else (50 if per_set < 4e9 else 10)
                        us = _time_events(torch, step, 3, iters)
                        byts = sum(decode_bytes(B, Hkv, d, ls, Hq) for ls in lens_sum) / nset
                        key = "parallax" if use_r else "softmax_only"
                        row[key + "_us"] = round(us, 2)
                        row[key + "_GBps"] = round(byts / us / 1e3, 1)
                    row["frac_of_8TBps"] = round(row["parallax_GBps"] / HBM_PEAK_GBPS, 4)
                    rows.append(row)
                    print("sweep", json.dumps(row), file=sys.stderr, flush=True)
                    del xs, al, o, w
    return {"metric": "decode_hbm_bandwidth_sweep", "unit": "GB/s", "n_gpus": 1, "dtype": "bf16",
            "data": "synthetic", "config": {"workload": "config3: decode sweep"}, "rows": rows}


def _preroll(torch, fn, seconds=PREROLL_SECONDS):
    """Run fn (untimed) until `seconds` of wall time have passed. After an idle gap -- input
    generation, a host-side pause -- the chip takes tens of milliseconds of load to bring its
    clocks up: a matrix-bound kernel measured in that window reads up to 15 % slow (the config-4
    prefill kernel: 493, 467, 456, 450 us at launches 1, 20, 40, 60 from idle, 448 us from then on
    for as long as it runs), an HBM-bound one about 1 %. Every timed loop below starts behind such
    a pre-roll of its own work, then its warm-up steps, then exactly the timed steps."""
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(4):
            fn()
        torch.cuda.synchronize()


def _time_events(torch, fn, warm, iters):
    _preroll(torch, fn)
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / iters  # microseconds


def extra_measurements(torch, plx, synth, lib, dev, sptr, sets, ws, out):
    """Decode sweep points (config 3, fixed-length grid), the softmax-only twin, the plain
    streaming-read ceiling, and causal prefill (config 4)."""
    extra = {}
    # achievable read bandwidth of a plain streaming kernel on this machine
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    sink = torch.empty(plx.parallax_util_read_sink_slots() * 16, dtype=torch.uint8, device=dev)
    us = _time_events(torch, lambda: plx.parallax_util_read(src, sink), 3, 20)
    extra["stream_read_ceiling_GBps"] = round(src.numel() / us / 1e3, 1)
    del src
    # sustained bf16 matrix rate of a register-only MFMA loop on this machine (one and four waves per SIMD)
    ceil = {}
    for wgs in (256, 1024):
        msink = torch.empty(wgs * 256, dtype=torch.float32, device=dev)
        flops = [0.0]

        def mstep():
            flops[0] = plx.parallax_util_mfma(wgs, 20000, msink)

        us = _time_events(torch, mstep, 1, 3)
        ceil["%d_workgroups_TFLOPs" % wgs] = round(flops[0] / us / 1e6, 1)
    ceil["frac_of_bf16_mfma_peak"] = round(max(ceil.values()) / MFMA_BF16_PEAK_TFLOPS, 4)
    extra["mfma_loop_ceiling"] = ceil

    # softmax-only twin on config 2
    x0 = sets
    twin_args = [plx.decode_args(x["q"], None, x["k"], x["v"], out, x["scale"], None, False, 0, ws)
                 for x in x0]
    cnt = [0]

    def twin():
        lib.parallax_decode(ctypes.byref(twin_args[cnt[0] % len(twin_args)]), sptr)
        cnt[0] += 1

    us = _time_events(torch, twin, 20, 200)
    extra["config2_softmax_only_us"] = round(us, 2)

    # config 2 with RMSNorm + RoPE on q, rho inside the decode kernel (weights, (cos, sin) table,
    # rows at position L - 1), interleaved with the plain step
    gam_q = 1.0 + 0.1 * torch.randn(128, device=dev)
    gam_r = 1.0 + 0.1 * torch.randn(128, device=dev)
    rtable = plx.parallax_rope_table(4096, 128, device=dev)
    prep_args = [plx.decode_args(x["q"], x["r"], x["k"], x["v"], out, x["scale"], None, True, 0, ws) for x in x0]
    for a in prep_args:
        a.prep = plx.qr_prep(gam_q, gam_r, rtable, None)
    plain_args = [plx.decode_args(x["q"], x["r"], x["k"], x["v"], out, x["scale"], None, True, 0, ws) for x in x0]

    def make(args):
        c = [0]

        def step():
            st = lib.parallax_decode(ctypes.byref(args[c[0] % len(args)]), sptr)
            c[0] += 1
            if st != 0:
                raise plx.ParallaxError(st, "decode with preparation")
        return step

    res = {"plain": [], "preparing": []}
    for _ in range(3):
        res["plain"].append(_time_events(torch, make(plain_args), 20, 200))
        res["preparing"].append(_time_events(torch, make(prep_args), 20, 200))
    extra["config2_decode_preparing_q_rho"] = {"plain_us": round(min(res["plain"]), 2),
                                               "preparing_us": round(min(res["preparing"]), 2)}

    # config 2 again as a HIP graph: the 8 rotated steps captured once, replayed (removes the
    # host's launch cost from the step time; every replay is the same 16 kernels)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g_args = [plx.decode_args(x["q"], x["r"], x["k"], x["v"], out, x["scale"], None, True, 0, ws)
              for x in x0]
    with torch.cuda.graph(graph, stream=side):
        cap = int(torch.cuda.current_stream().cuda_stream)
        for a in g_args:
            st = lib.parallax_decode(ctypes.byref(a), cap)
            if st != 0:
                raise plx.ParallaxError(st, "graph capture")
    torch.cuda.current_stream().wait_stream(side)
    us = _time_events(torch, graph.replay, 5, 50) / len(g_args)
    extra["config2_hip_graph_replay_us_per_step"] = round(us, 2)

    # config 2 with the merge inside the split kernel (one launch per step), interleaved with
    # the two-kernel path so that both see the same clocks
    counters = torch.zeros(64, dtype=torch.int32, device=dev)
    f_args = [plx.decode_args(x["q"], x["r"], x["k"], x["v"], out, x["scale"], None, True, 0, ws)
              for x in x0]
    for a in f_args:
        a.split_counters = counters.data_ptr()
    fc = [0]

    def fused_step():
        lib.parallax_decode_fused(ctypes.byref(f_args[fc[0] % len(f_args)]), sptr)
        fc[0] += 1

    def plain_step():
        lib.parallax_decode(ctypes.byref(g_args[fc[0] % len(g_args)]), sptr)
        fc[0] += 1

    pair = [[], []]
    for _ in range(3):
        pair[0].append(_time_events(torch, plain_step, 20, 200))
        pair[1].append(_time_events(torch, fused_step, 20, 200))
    fused = {"config2": {"two_kernels_us": round(min(pair[0]), 2), "one_kernel_us": round(min(pair[1]), 2)}}
    # ... and where the launch boundary weighs most (one sequence) or the merge is widest
    # (several query rows: 8 merged rows per group)
    for name, (B, L, Tq) in (("B1_L8192", (1, 8192, 1)), ("B4_L16384_Tq4", (4, 16384, 4))):
        xs = [synth.decode_inputs(B, 16, 8, L, 128, seed=3300 + i, device=dev) for i in range(4)]
        if Tq > 1:
            qr = synth.prefill_inputs(B, 16, 8, Tq, 128, seed=3310, device=dev)
            for x in xs:
                x["q"], x["r"] = qr["q"].contiguous(), qr["r"].contiguous()
        o2 = torch.empty_like(xs[0]["q"])
        ws2 = torch.empty(plx.parallax_decode_workspace_bytes(B, 16 * Tq, 8, L, 128) // 4,
                          dtype=torch.float32, device=dev)
        s_args = [plx.decode_args(x["q"], x["r"], x["k"], x["v"], o2, x["scale"], None, True, 0, ws2)
                  for x in xs]
        for a in s_args:
            a.split_counters = counters.data_ptr()
        sc = [0]

        def step(entry):
            st = entry(ctypes.byref(s_args[sc[0] % len(s_args)]), sptr)
            sc[0] += 1
            if st != 0:
                raise plx.ParallaxError(st, "in-kernel reduction bench")

        t2, t1 = [], []
        for _ in range(3):
            t2.append(_time_events(torch, lambda: step(lib.parallax_decode), 20, 200))
            t1.append(_time_events(torch, lambda: step(lib.parallax_decode_fused), 20, 200))
        fused[name] = {"two_kernels_us": round(min(t2), 2), "one_kernel_us": round(min(t1), 2)}
        del xs, s_args, ws2
    extra["in_kernel_reduction"] = fused

    # config 2 behind a block table (paged cache, shuffled page pool), 8 rotated pools
    paged = {}
    for page_size in (16, 128):
        pools = [synth.paged_cache(x, page_size, seed=7000 + i) for i, x in enumerate(x0)]
        p_args = [plx.decode_args(x["q"], x["r"], kp, vp, out, x["scale"], None, True, 0, ws,
                                  block_table=tb, max_len=x["k"].shape[2])
                  for x, (kp, vp, tb) in zip(x0, pools)]
        pc = [0]

        def paged_step():
            lib.parallax_decode(ctypes.byref(p_args[pc[0] % len(p_args)]), sptr)
            pc[0] += 1

        paged["page_size_%d_us" % page_size] = round(_time_events(torch, paged_step, 20, 200), 2)
        del pools, p_args
    extra["config2_paged_cache"] = paged

    # several query rows per sequence (speculative rows): same K/V traffic as one row
    multi = []
    for (B, L, Tq) in [(64, 4096, 4), (64, 4096, 8), (8, 16384, 4)]:
        Hq, Hkv, d = 16, 8, 128
        per_set = B * Hkv * L * d * 4
        nset = max(1, min(8, int(1.2e9 // per_set) + 1))
        xs = [synth.decode_inputs(B, Hq, Hkv, L, d, seed=3100 + i, device=dev) for i in range(nset)]
        qr = synth.prefill_inputs(B, Hq, Hkv, Tq, d, seed=3200, device=dev)
        o = torch.empty_like(qr["q"])
        w = torch.empty(Tq * plx.parallax_decode_workspace_bytes(B, Hq, Hkv, L, d) // 4,
                        dtype=torch.float32, device=dev)
        al = [plx.decode_args(qr["q"], qr["r"], x["k"], x["v"], o, x["scale"], None, True, 0, w)
              for x in xs]
        mc = [0]

        def multi_step():
            lib.parallax_decode(ctypes.byref(al[mc[0] % nset]), sptr)
            mc[0] += 1

        us = _time_events(torch, multi_step, 5, 50)
        multi.append({"B": B, "L": L, "Tq": Tq, "us": round(us, 2),
                      "kv_GBps": round(per_set / us / 1e3, 1)})
        del xs, al
    extra["decode_several_query_rows"] = multi

    sweep = []
    for (B, L) in [(1, 1024), (1, 65536), (16, 4096), (16, 16384), (64, 16384), (128, 16384)]:
        Hq, Hkv, d = 16, 8, 128
        per_set = B * Hkv * L * d * 4
        nset = max(1, min(8, int(3e9 // per_set)))
        xs = [synth.decode_inputs(B, Hq, Hkv, L, d, seed=3000 + i, device=dev) for i in range(nset)]
        o = torch.empty_like(xs[0]["q"])
        w = torch.empty(plx.parallax_decode_workspace_bytes(B, Hq, Hkv, L, d) // 4,
                        dtype=torch.float32, device=dev)
        row = {"B": B, "L": L, "num_splits": plx.parallax_decode_num_splits(B, Hq, Hkv, L, d),
               "kv_sets": nset}
        for use_r in (True, False):
            al = [plx.decode_args(x["q"], x["r"], x["k"], x["v"], o, x["scale"], None, use_r, 0, w)
                  for x in xs]
            c = [0]

            def step():
                lib.parallax_decode(ctypes.byref(al[c[0] % nset]), sptr)
                c[0] += 1

            iters = 200 if per_set < 5e8 else 30
            us = _time_events(torch, step, 5, iters)
            byts = decode_bytes(B, Hkv, d, B * L, Hq)
            key = "parallax" if use_r else "softmax_only"
            row[key + "_us"] = round(us, 2)
            row[key + "_GBps"] = round(byts / us / 1e3, 1)
        row["frac_of_8TBps"] = round(row["parallax_GBps"] / HBM_PEAK_GBPS, 4)
        sweep.append(row)
        del xs, al
    extra["decode_sweep"] = sweep

    # Few sequences at long context (the region where a step is short enough for launch and ramp
    # to weigh): B in {1, 8} x L in {8192, 16384, 65536}, fixed and ragged lengths, each next to
    # the best a plain read kernel does on the same number of bytes on this machine (grids of 256 ...
    # 4096 workgroups; 256 = one persistent workgroup per compute unit), rotating over a 1.6 GB
    # buffer so that nothing is found in the Infinity Cache. And config 5b (B = 32, L = 131072).
    big = torch.empty(1600 << 20, dtype=torch.uint8, device=dev).zero_()
    floor_cache = {}

    def read_floor_us(nbytes):
        nbytes = (int(nbytes) + 4095) // 4096 * 4096
        if nbytes not in floor_cache:
            span = max(1, (big.numel() - nbytes) // 4096)
            best = None
            for wgs in (256, 512, 1024, 2048, 4096):
                k = [0]

                def rstep():
                    off = (k[0] * 977 % span) * 4096 if nbytes < big.numel() else 0
                    plx.parallax_util_read_grid(big[off:], sink, wgs, nbytes=min(nbytes, big.numel()))
                    k[0] += 1

                us = _time_events(torch, rstep, 5, 60)
                if best is None or us < best[0]:
                    best = (us, wgs)
            floor_cache[nbytes] = best
        return floor_cache[nbytes]

    small = []
    for (B, L) in [(1, 8192), (1, 16384), (1, 65536), (8, 8192), (8, 16384), (8, 65536), (32, 131072)]:
        Hq, Hkv, d = 16, 8, 128
        per_set = B * Hkv * L * d * 4
        nset = max(1, min(8, int(2.2e9 // per_set)))
        for ragged in ((False, True) if L < 131072 else (False,)):
            xs = [synth.decode_inputs(B, Hq, Hkv, L, d, seed=3400 + i, device=dev, ragged=ragged,
                                      r_scale=0.1 if L == 131072 else 1.0) for i in range(nset)]
            o = torch.empty_like(xs[0]["q"])
            w = torch.empty(plx.parallax_decode_workspace_bytes(B, Hq, Hkv, L, d) // 4,
                            dtype=torch.float32, device=dev)
            al = [plx.decode_args(x["q"], x["r"], x["k"], x["v"], o, x["scale"], x.get("seq_lens"), True, 0, w)
                  for x in xs]
            c = [0]

            def step():
                lib.parallax_decode(ctypes.byref(al[c[0] % nset]), sptr)
                c[0] += 1

            us = _time_events(torch, step, 5, 200 if per_set < 5e8 else 20)
            byts = sum(decode_bytes(B, Hkv, d, int(x["seq_lens"].sum().item()) if ragged else B * L, Hq)
                       for x in xs) / nset
            row = {"B": B, "L": L, "ragged": ragged, "kv_sets": nset,
                   "num_splits": plx.parallax_decode_num_splits(B, Hq, Hkv, L, d),
                   "us": round(us, 2), "GBps": round(byts / us / 1e3, 1),
                   "frac_of_8TBps": round(byts / us / 1e3 / HBM_PEAK_GBPS, 4)}
            if per_set <= big.numel():
                f_us, f_wgs = read_floor_us(byts)
                row["plain_read_same_bytes_us"] = round(f_us, 2)
                row["plain_read_workgroups"] = f_wgs
                row["step_over_plain_read"] = round(us / f_us, 3)
            if L == 131072:
                row["workload"] = "config5b: decode bf16 B=32 L=131072, R x0.1"
            small.append(row)
            del xs, al, o, w
    extra["decode_few_sequences_long_context"] = small
    f_us, f_wgs = read_floor_us(decode_bytes(8, 8, 128, 8 * 4096, 16))
    extra["config2_plain_read_same_bytes"] = {"us": round(f_us, 2), "workgroups": f_wgs}
    del big

    # causal prefill, config 4
    B, T, Hq, Hkv, d = 4, 4096, 16, 8, 128
    y = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=1004, device=dev, k_offset_sigma=0.5)
    po = torch.empty_like(y["q"])
    pre = {}
    for use_r in (True, False):
        us = _time_events(
            torch, lambda: plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"],
                                                causal=True, use_r=use_r, out=po), 3, 20)
        flops = B * Hq * (8 if use_r else 4) * d * T * (T + 1) / 2
        key = "parallax" if use_r else "softmax_only"
        pre[key + "_us"] = round(us, 1)
        pre[key + "_TFLOPs"] = round(flops / us / 1e6, 1)
    pre["frac_of_bf16_mfma_peak"] = round(pre["parallax_TFLOPs"] / MFMA_BF16_PEAK_TFLOPS, 4)
    pre["frac_of_mfma_loop_ceiling"] = round(
        pre["parallax_TFLOPs"] / max(v for k, v in extra["mfma_loop_ceiling"].items() if k.endswith("TFLOPs")), 4)
    pre["workload"] = "config4: causal prefill bf16 B=4 T=4096 Hq=16 Hkv=8 d=128, K offset N(0,0.5^2)"
    extra["prefill"] = pre
    # ... and its backward pass (rows prepare + dQ/dR pass + dK/dV pass; 22 d flops per pair)
    g = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=1014, device=dev)["q"].contiguous()
    o, vbar, stats = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=True,
                                          save_for_backward=True)
    bws = torch.empty(plx.parallax_prefill_backward_workspace_bytes(B, Hq, T) // 4,
                      dtype=torch.float32, device=dev)
    us = _time_events(
        torch, lambda: plx.parallax_prefill_backward(y["q"], y["r"], y["k"], y["v"], o, vbar, stats, g,
                                                     y["scale"], causal=True, workspace=bws), 2, 10)
    bflops = B * Hq * 22 * d * T * (T + 1) / 2
    extra["prefill_backward"] = {
        "workload": "backward of config 4 (causal B=4 T=4096 d=128)", "us": round(us, 1),
        "TFLOPs": round(bflops / us / 1e6, 1),
        "frac_of_bf16_mfma_peak": round(bflops / us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4)}
    del y, po, g, o, vbar, stats, bws

    # other prefill shapes: config 5a (long causal), full attention, and the compute-matched
    # d = 64 layout (twice the heads, half the head dimension)
    more = []
    for (name, B, T, Hq, Hkv, d, causal, r_scale) in [
            ("config5a: causal B=2 T=16384 d=128, R x0.1", 2, 16384, 16, 8, 128, True, 0.1),
            ("full attention B=4 T=4096 d=128", 4, 4096, 16, 8, 128, False, 1.0),
            ("causal B=4 T=4096 d=64, 32 query / 16 KV heads", 4, 4096, 32, 16, 64, True, 1.0)]:
        y = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=1005, device=dev, r_scale=r_scale)
        po = torch.empty_like(y["q"])
        us = _time_events(
            torch, lambda: plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"],
                                                causal=causal, out=po), 2, 10)
        flops = B * Hq * 8 * d * (T * (T + 1) / 2 if causal else T * T)
        more.append({"workload": name, "us": round(us, 1), "TFLOPs": round(flops / us / 1e6, 1),
                     "frac_of_bf16_mfma_peak": round(flops / us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4)})
        del y, po
    # chunked prefill: T new rows behind an existing cache (causal, rows = the last T positions)
    for (B, T, Tkv) in [(8, 512, 8192), (4, 2048, 16384), (64, 4, 4096)]:
        Hq, Hkv, d = 16, 8, 128
        y = synth.prefill_inputs(B, Hq, Hkv, Tkv, d, seed=1006, device=dev)
        qc, rc = y["q"][:, :, -T:].contiguous(), y["r"][:, :, -T:].contiguous()
        po = torch.empty_like(qc)
        us = _time_events(
            torch, lambda: plx.parallax_prefill(qc, rc, y["k"], y["v"], y["scale"], causal=True,
                                                out=po), 2, 10)
        pairs = T * (Tkv - T) + T * (T + 1) / 2  # allowed (row, key) pairs per head
        flops = B * Hq * 8 * d * pairs
        more.append({"workload": "chunked causal B=%d T=%d rows over Tkv=%d keys, d=128" % (B, T, Tkv),
                     "us": round(us, 1), "TFLOPs": round(flops / us / 1e6, 1),
                     "frac_of_bf16_mfma_peak": round(flops / us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4),
                     "kv_GBps": round(B * Hkv * Tkv * d * 4 / us / 1e3, 1)})
        del y, po, qc, rc
    extra["prefill_more"] = more

    # RMSNorm + RoPE on q, rho, k of the config-4 shape in one launch (read once, written once)
    B, T, Hq, Hkv, d = 4, 4096, 16, 8, 128
    y = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=1009, device=dev)
    gam = [torch.ones(d, dtype=torch.float32, device=dev) for _ in range(3)]
    outs = [torch.empty_like(y[n]) for n in ("q", "r", "k")]
    na = plx.norm_rope_args([(y["q"], gam[0], True, outs[0]), (y["r"], gam[1], True, outs[1]),
                             (y["k"], gam[2], True, outs[2])])

    def nr_step():
        st = lib.parallax_norm_rope(ctypes.byref(na), sptr)
        if st != 0:
            raise plx.ParallaxError(st, "parallax_norm_rope")

    us = _time_events(torch, nr_step, 5, 50)
    nbytes = 2 * sum(t.numel() * 2 for t in outs)
    extra["norm_rope"] = {"workload": "RMSNorm + RoPE on q, rho [4,16,4096,128] and k [4,8,4096,128] bf16, one launch",
                          "us": round(us, 1), "GBps": round(nbytes / us / 1e3, 1),
                          "frac_of_8TBps": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4)}
    # the same preparation of q and rho inside the prefill kernel (k alone goes through the
    # launch above): bare prefill on prepared inputs / the two-launch chain / fused
    po = torch.empty_like(y["q"])
    table = plx.parallax_rope_table(T, d, device=dev)
    na_k = plx.norm_rope_args([(y["k"], gam[2], True, outs[2])])
    a_bare = plx.prefill_args(outs[0], outs[1], outs[2], y["v"], po, y["scale"], True, True)
    a_fused = plx.prefill_args(y["q"], y["r"], outs[2], y["v"], po, y["scale"], True, True)
    a_fused.prep = plx.qr_prep(gam[0], gam[1], table, None)

    def call(fn, args):
        st = fn(ctypes.byref(args), sptr)
        if st != 0:
            raise plx.ParallaxError(st, "fused preparation")

    variants = {"prefill_on_prepared_inputs_us": lambda: call(lib.parallax_prefill, a_bare),
                "norm_rope_qrk_then_prefill_us": lambda: (call(lib.parallax_norm_rope, na), call(lib.parallax_prefill, a_bare)),
                "norm_rope_k_then_prefill_preparing_q_rho_us": lambda: (call(lib.parallax_norm_rope, na_k),
                                                                        call(lib.parallax_prefill, a_fused)),
                "prefill_preparing_q_rho_us": lambda: call(lib.parallax_prefill, a_fused)}
    fz = {"workload": "config-4 shape [4,16/8,4096,128] bf16 causal; RMSNorm + RoPE (theta 1e6) on q, rho, k"}
    for name, fn in variants.items():
        fz[name] = round(_time_events(torch, fn, 3, 20), 1)
    fz["in_kernel_preparation_over_bare_prefill"] = round(
        fz["prefill_preparing_q_rho_us"] / fz["prefill_on_prepared_inputs_us"] - 1.0, 4)
    extra["norm_rope_fused_into_prefill"] = fz
    del y, outs, po

    # sliding window (a row sees its own position and the window - 1 before it)
    win = []
    for (B, T, W) in [(2, 16384, 4096), (2, 16384, 1024)]:
        Hq, Hkv, d = 16, 8, 128
        y = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=1007, device=dev)
        po = torch.empty_like(y["q"])
        us = _time_events(
            torch, lambda: plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"],
                                                causal=True, out=po, window=W), 2, 10)
        pairs = W * (W + 1) / 2 + (T - W) * W  # allowed (row, key) pairs per head
        flops = B * Hq * 8 * d * pairs
        win.append({"workload": "causal prefill B=%d T=%d window=%d d=128" % (B, T, W),
                    "us": round(us, 1), "TFLOPs": round(flops / us / 1e6, 1),
                    "frac_of_bf16_mfma_peak": round(flops / us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4)})
        # ... and its backward (22 d flops per allowed pair)
        g = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=1015, device=dev)["q"].contiguous()
        o, vbar, stats = plx.parallax_prefill(y["q"], y["r"], y["k"], y["v"], y["scale"], causal=True,
                                              save_for_backward=True, window=W)
        bws = torch.empty(plx.parallax_prefill_backward_workspace_bytes(B, Hq, T) // 4,
                          dtype=torch.float32, device=dev)
        us = _time_events(
            torch, lambda: plx.parallax_prefill_backward(y["q"], y["r"], y["k"], y["v"], o, vbar, stats, g,
                                                         y["scale"], causal=True, workspace=bws, window=W), 2, 5)
        bflops = B * Hq * 22 * d * pairs
        win.append({"workload": "backward of causal prefill B=%d T=%d window=%d d=128" % (B, T, W),
                    "us": round(us, 1), "TFLOPs": round(bflops / us / 1e6, 1),
                    "frac_of_bf16_mfma_peak": round(bflops / us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4)})
        del y, po, g, o, vbar, stats, bws
    for (B, L, W) in [(16, 65536, 4096), (16, 4096, 0)]:
        Hq, Hkv, d = 16, 8, 128
        xs = [synth.decode_inputs(B, Hq, Hkv, L, d, seed=1008 + i, device=dev)
              for i in range(2 if L > 4096 else 8)]
        o2 = torch.empty_like(xs[0]["q"])
        ws2 = torch.empty(plx.parallax_decode_workspace_bytes(B, Hq, Hkv, L, d) // 4,
                          dtype=torch.float32, device=dev)
        w_args = [plx.decode_args(x["q"], x["r"], x["k"], x["v"], o2, x["scale"], None, True, 0, ws2,
                                  window=W) for x in xs]
        wc = [0]

        def wstep():
            st = lib.parallax_decode(ctypes.byref(w_args[wc[0] % len(w_args)]), sptr)
            wc[0] += 1
            if st != 0:
                raise plx.ParallaxError(st, "window bench")

        us = _time_events(torch, wstep, 20, 200)
        keys = min(L, W) if W else L
        win.append({"workload": "decode B=%d L=%d window=%d d=128" % (B, L, W), "us": round(us, 2),
                    "kv_GBps_of_keys_in_window": round(B * Hkv * keys * d * 4 / us / 1e3, 1)})
        del xs, w_args, ws2
    extra["sliding_window"] = win

    # block-sparse prefill: each 128-row block visits a listed subset of the 64-key tiles
    # (flops = 8 d per allowed (row, key) pair inside the listed tiles, intersected with the causal set)
    import numpy as np

    bs = []
    for (B, T) in [(4, 4096), (2, 16384)]:
        Hq, Hkv, d = 16, 8, 128
        y = synth.prefill_inputs(B, Hq, Hkv, T, d, seed=1010, device=dev)
        po = torch.empty_like(y["q"])
        nrb, nkt = T // plx.BLOCK_ROWS, T // plx.BLOCK_KEYS
        diag = 2 * np.arange(nrb)[:, None] + 1                  # last tile a row block can see
        band = (np.arange(nkt)[None, :] > diag - 32) | (np.arange(nkt)[None, :] < 4)
        rnd = np.random.default_rng(1011).random((nrb, nkt)) < 0.25
        for name, bm in [("every causal tile", np.ones((nrb, nkt), bool)),
                         ("band of 32 tiles + first 4", band), ("random 25% of tiles", rnd)]:
            bm = bm & (np.arange(nkt)[None, :] <= diag)
            row_ptr, tile_idx, Bs, Hs = plx.block_mask_lists(torch.as_tensor(bm, device=dev))
            a = plx.prefill_args(y["q"], y["r"], y["k"], y["v"], po, y["scale"], True, True)
            a.sparse_row_ptr, a.sparse_tile_idx = row_ptr.data_ptr(), tile_idx.data_ptr()
            a.sparse_batch, a.sparse_heads = Bs, Hs

            def sstep():
                st = lib.parallax_prefill(ctypes.byref(a), sptr)
                if st != 0:
                    raise plx.ParallaxError(st, "block-sparse bench")

            us = _time_events(torch, sstep, 2, 10)
            # a listed tile strictly below the diagonal holds 128 * 64 pairs; the two on it 64 * 65 / 2
            # + 64 * 64 and 64 * 65 / 2 (row block i: tiles 2i and 2i + 1)
            below = int((bm & (np.arange(nkt)[None, :] < diag - 1)).sum())
            on_lo = int(bm[np.arange(nrb), 2 * np.arange(nrb)].sum())
            on_hi = int(bm[np.arange(nrb), 2 * np.arange(nrb) + 1].sum())
            pairs = below * 128 * 64 + on_lo * (64 * 65 // 2 + 64 * 64) + on_hi * (64 * 65 // 2)
            flops = B * Hq * 8 * d * pairs
            rec = {"workload": "block-sparse causal prefill B=%d T=%d d=128, %s" % (B, T, name),
                   "tiles_listed": int(bm.sum()), "tiles_causal": int((np.arange(nkt)[None, :] <= diag).sum()),
                   "us": round(us, 1), "TFLOPs": round(flops / us / 1e6, 1),
                   "frac_of_bf16_mfma_peak": round(flops / us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4)}
            if B == 4:
                # the backward over the same lists (three kernels; 22 d flops per allowed pair)
                vbar = torch.empty_like(po)
                stats = torch.empty(B, Hq, T, 2, dtype=torch.float32, device=dev)
                a.vbar, a.row_stats = vbar.data_ptr(), stats.data_ptr()
                sstep()
                col_ptr, col_idx = plx.block_mask_column_lists(torch.as_tensor(bm, device=dev))
                grads = [torch.empty_like(y[n]) for n in ("q", "r", "k", "v")]
                bws = torch.empty(B * Hq * T * 4, dtype=torch.float32, device=dev)
                ba = plx.prefill_bwd_args(y["q"], y["r"], y["k"], y["v"], po, vbar, stats, y["q"], *grads,
                                          y["scale"], True, bws)
                ba.sparse_row_ptr, ba.sparse_tile_idx = row_ptr.data_ptr(), tile_idx.data_ptr()
                ba.sparse_col_ptr, ba.sparse_col_idx = col_ptr.data_ptr(), col_idx.data_ptr()
                ba.sparse_batch, ba.sparse_heads = Bs, Hs

                def bstep():
                    st = lib.parallax_prefill_backward(ctypes.byref(ba), sptr)
                    if st != 0:
                        raise plx.ParallaxError(st, "block-sparse backward bench")

                bus = _time_events(torch, bstep, 2, 10)
                bflops = B * Hq * 22 * d * pairs
                rec["backward_us"] = round(bus, 1)
                rec["backward_frac_of_bf16_mfma_peak"] = round(bflops / bus / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4)
                a.vbar, a.row_stats = None, None
                del vbar, stats, grads, bws
            bs.append(rec)
        del y, po
    extra["block_sparse"] = bs

    # decode over an MLA-style latent cache: one row of 512 + 64 numbers per token, shared by all
    # heads (algorithmic bytes: the cache once, q, r, o)
    ml = []
    for (B, Hq, L) in [(64, 16, 16384), (32, 16, 8192), (128, 16, 4096), (16, 128, 8192)]:
        nset = max(2, min(8, int(2e9 // (B * L * 1152))))
        xs = [synth.mla_decode_inputs(B, Hq, L, seed=1012 + i, device=dev) for i in range(nset)]
        mo = torch.empty(B, Hq, 512, dtype=torch.bfloat16, device=dev)
        mws = torch.empty(plx.parallax_decode_mla_workspace_bytes(B, Hq) // 4, dtype=torch.float32, device=dev)
        m_args = [plx.decode_mla_args(x["q"], x["r"], x["ckv"], mo, x["scale"], None, 0, mws) for x in xs]
        mc = [0]

        def mstep2():
            st = lib.parallax_decode_mla(ctypes.byref(m_args[mc[0] % nset]), sptr)
            mc[0] += 1
            if st != 0:
                raise plx.ParallaxError(st, "mla bench")

        us = _time_events(torch, mstep2, 5, 50)
        nbytes = B * L * 1152 + B * Hq * (2 * 576 * 2 + 512 * 2)
        ml.append({"workload": "MLA-style decode B=%d Hq=%d L=%d (latent 512 + rope 64)" % (B, Hq, L),
                   "num_splits": plx.parallax_decode_mla_num_splits(B, Hq, L), "us": round(us, 1),
                   "GBps": round(nbytes / us / 1e3, 1), "frac_of_8TBps": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4),
                   "TFLOPs": round(B * Hq * L * 2 * (2 * 576 + 2 * 512) / us / 1e6, 1)})
        if (B, L) == (64, 16384):  # the same tokens behind a block table, pages of 256 tokens in random order
            pools = [synth.mla_paged_cache(x, 256, seed=1013 + i) for i, x in enumerate(xs)]
            p_args = [plx.decode_mla_args(x["q"], x["r"], pool, mo, x["scale"], None, 0, mws, block_table=table,
                                          max_len=L) for x, (pool, table) in zip(xs, pools)]

            def pstep():
                st = lib.parallax_decode_mla(ctypes.byref(p_args[mc[0] % nset]), sptr)
                mc[0] += 1
                if st != 0:
                    raise plx.ParallaxError(st, "paged mla bench")

            us = _time_events(torch, pstep, 5, 50)
            ml.append({"workload": "MLA-style decode B=%d Hq=%d L=%d, paged cache (256 tokens per page)" % (B, Hq, L),
                       "us": round(us, 1), "GBps": round(nbytes / us / 1e3, 1),
                       "frac_of_8TBps": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4)})
            del pools, p_args
        del xs, m_args, mo, mws
    extra["mla_decode"] = ml

    # several rows per head over the latent cache: a 4-row decode step, and the causal prefill
    # (rows = prompt; flops = 4352 per (head, row, visible token), bytes = the cache once per batch entry)
    mr = []
    for (B, Hq, Tq, L) in [(64, 16, 4, 16384), (2, 16, 4096, 4096)]:
        x = synth.mla_decode_inputs(B, Hq * Tq, L, seed=1030, device=dev)
        q4, r4 = x["q"].view(B, Hq, Tq, 576), x["r"].view(B, Hq, Tq, 576)
        mo = torch.empty(B, Hq, Tq, 512, dtype=torch.bfloat16, device=dev)
        S = plx.parallax_decode_mla_num_splits(B, Hq * Tq, L)
        mws = torch.empty(max(B * Hq * Tq * S * 1028, 4), dtype=torch.float32, device=dev)
        ma = plx.decode_mla_args(q4, r4, x["ckv"], mo, x["scale"], None, S, mws)

        def rstep():
            st = lib.parallax_decode_mla(ctypes.byref(ma), sptr)
            if st != 0:
                raise plx.ParallaxError(st, "mla rows bench")

        us = _time_events(torch, rstep, 2, 10)
        pairs = B * Hq * sum(L - Tq + t + 1 for t in range(Tq))
        mr.append({"workload": "latent cache, B=%d Hq=%d, %d rows per head at the end of L=%d" % (B, Hq, Tq, L),
                   "num_splits": S, "us": round(us, 1), "TFLOPs": round(4352.0 * pairs / us / 1e6, 1),
                   "cache_GBps": round(B * L * 1152 / us / 1e3, 1)})
        del x, mo, mws
    extra["mla_rows"] = mr
    return extra


if __name__ == "__main__":
    main()
