"""bench.py pieces that need no GPU: the byte accounting and the one-GPU guard."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_decode_bytes_counts_k_and_v_once_plus_q_r_o():
    sys.path.insert(0, ROOT)
    import bench

    # config 2: 8 sequences x 4096 keys, 8 KV heads, d = 128, bf16: 4096 bytes per cached token
    B, Hq, Hkv, L, d = 8, 16, 8, 4096, 128
    assert bench.decode_bytes(B, Hkv, d, B * L, Hq) == B * L * 4096 + 3 * B * Hq * d * 2 == 134316032


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=120)
    assert res.returncode == 2
    assert "one GPU" in res.stderr and res.stdout.strip() == ""


def _write_csv(path, header, rows):
    with open(path, "w") as f:
        f.write(",".join(header) + "\n")
        for r in rows:
            f.write(",".join('"%s"' % x if isinstance(x, str) else str(x) for x in r) + "\n")


def test_profiling_summaries_from_rocprofv3_csv(tmp_path, capsys):
    """profiling.py (host only): trace statistics with the last K dispatches listed apart, and
    HBM traffic = counter reading x what the same counter reads for the copy of known size."""
    sys.path.insert(0, ROOT)
    from paper_2605_29157_amd import profiling

    trace = str(tmp_path / "t_kernel_trace.csv")
    rows = [("void plx::attn_kernel<128>(plx::P)", 1000 * i, 1000 * i + (900 if i < 4 else 500)) for i in range(10)]
    rows.append(("void other_kernel()", 50000, 50010))
    _write_csv(trace, ["Kernel_Name", "Start_Timestamp", "End_Timestamp"], rows)
    tr = profiling.read_trace(trace)
    assert tr["void attn_kernel<128>"] == [0.9] * 4 + [0.5] * 6
    profiling.main(["trace", trace, "--kernel", "attn_kernel", "--last", "6"])
    out = capsys.readouterr().out
    assert "| `void attn_kernel<128>` | 10 | 0.66 | 0.50 | 0.50 | 0.90 |" in out
    assert "last 6 dispatches" in out and "mean 0.50 us" in out

    def counters(path, counter, copy_kib, kernel_kib):
        rows = []
        for d in range(3):  # two instances per dispatch: they add up
            rows += [("void plx::util_copy_kernel(a)", counter, d, copy_kib / 2)] * 2
        for d in range(3, 7):
            rows += [("void plx::attn_kernel<128>(plx::P)", counter, d, kernel_kib)]
        _write_csv(path, ["Kernel_Name", "Counter_Name", "Dispatch_Id", "Counter_Value"], rows)

    fetch, write = str(tmp_path / "f.csv"), str(tmp_path / "w.csv")
    counters(fetch, "FETCH_SIZE", 512.0, 100.0)     # the counter reads half of the bytes fetched
    counters(write, "WRITE_SIZE", 1024.0, 10.0)
    traffic = str(tmp_path / "traffic.txt")
    with open(traffic, "w") as f:
        f.write("# kept\nother_key = 7\n")
    profiling.main(["traffic", "--fetch", fetch, "--write", write, "--kernel", "attn_kernel",
                    "--copy-bytes", str(1024 * 1024), "--key", "attn", "--out", traffic])
    vals = profiling.read_traffic_file(traffic)
    assert vals == {"other_key": 7, "attn": (100 * 2 + 10) * 1024}
    import bench

    old = bench.TRAFFIC_FILE
    try:
        bench.TRAFFIC_FILE = traffic
        assert bench.measured_traffic("attn") == 215040 and bench.measured_traffic("missing") is None
    finally:
        bench.TRAFFIC_FILE = old
