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
