"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_2605_29157_amd import binding as b

    if not os.path.exists(b.LIB_PATH):
        from paper_2605_29157_amd import build

        build.build_library(verbose=False)
    b.load_library()
    return b


def _declared_functions():
    """Every function declared by the headers under include/ (the attention ABI and the
    measurement helpers)."""
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(parallax_\w+)\s*\(", text))
    return sorted(names)


def test_header_symbols_are_exported(binding):
    names = _declared_functions()
    assert len(names) >= 9
    lib = binding.load_library()
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTED_SYMBOLS) == names


def test_struct_sizes_match_c_layout(binding):
    # 6 pointers, 5 int32 (+pad), 6 int64, float + 2 int32 (+pad), pointer, size_t, enum (+pad),
    # pointer, 4 int32, int32 (+pad), pointer, the q / rho preparation (4 pointers, 3 int32, float)
    assert ctypes.sizeof(binding.plx_qr_prep) == 4 * 8 + 16
    assert ctypes.sizeof(binding.plx_decode_args) == 6 * 8 + 24 + 6 * 8 + 16 + 8 + 8 + 8 + 8 + 16 + 8 + 8 + 48
    # 5 pointers, 5 int32 (+pad), 15 int64, float + 2 int32 + enum, 2 int32, 2 pointers
    assert ctypes.sizeof(binding.plx_prefill_args) == 5 * 8 + 24 + 15 * 8 + 16 + 8 + 16 + 16 + 8 + 48
    # 12 pointers, 6 int32, float + int32, enum (+pad), pointer, size_t, 11 stride triples,
    # 4 list pointers, 2 int32
    assert ctypes.sizeof(binding.plx_prefill_bwd_args) == 12 * 8 + 24 + 8 + 8 + 16 + 11 * 24 + 4 * 8 + 8


def test_struct_layouts_match_a_c_compiler(binding, tmp_path):
    """sizeof and every field offset of the ctypes mirrors against gcc's reading of the header."""
    import subprocess

    structs = ["plx_qr_prep", "plx_decode_args", "plx_prefill_args", "plx_prefill_bwd_args", "plx_norm_rope_tensor",
               "plx_norm_rope_args", "plx_decode_mla_args"]
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "parallax.h"', 'int main(void) {']
    for sname in structs:
        lines.append('printf("%s %%zu\\n", sizeof(%s));' % (sname, sname))
        for f in getattr(binding, sname)._fields_:
            lines.append('printf("%s.%s %%zu\\n", offsetof(%s, %s));' % (sname, f[0], sname, f[0]))
    lines += ['return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    want = dict(l.split() for l in out if l)
    for sname in structs:
        cls = getattr(binding, sname)
        assert ctypes.sizeof(cls) == int(want[sname]), sname
        for f in cls._fields_:
            assert getattr(cls, f[0]).offset == int(want["%s.%s" % (sname, f[0])]), (sname, f[0])


def test_version_and_strerror(binding):
    assert binding.version() >= 100
    assert binding.strerror(0) == "ok"
    for code in range(-9, 0):
        assert binding.strerror(code) not in ("ok", "unknown status")
    assert binding.strerror(-99) == "unknown status"


def test_workspace_bytes(binding):
    n = binding.parallax_decode_workspace_bytes(8, 16, 8, 4096, 128)
    assert n == 8 * 16 * binding.PLX_MAX_SPLITS * (2 * 128 + 4) * 4
    assert binding.parallax_decode_workspace_bytes(0, 16, 8, 4096, 128) == 0


def test_split_heuristic_is_sane(binding):
    f = binding.parallax_decode_num_splits
    # explicit CU count: pure host arithmetic
    for (B, L) in [(1, 1024), (8, 4096), (16, 16384), (128, 65536), (32, 131072), (1, 1), (2, 100)]:
        s = f(B, 16, 8, L, 128, 256)
        assert 1 <= s <= binding.PLX_MAX_SPLITS
        n_bt = (L + 127) // 128
        assert s <= max(1, n_bt // 2)          # at least two block tiles per split
    assert f(8, 16, 8, 4096, 128, 256) == 8    # 512 workgroups over 64 (batch, kv head) pairs
    assert f(1, 16, 8, 256, 128, 256) == 1
    assert f(1, 16, 8, 512, 128, 256) == 1     # no split below 1024 keys
    assert f(1, 16, 8, 1024, 128, 256) == 4
    # enough pairs to keep every compute unit reading: no split, or a whole number of rounds
    assert f(16, 16, 8, 2048, 128, 256) == 1
    assert f(16, 16, 8, 16384, 128, 256) == 4  # 512 workgroups
    assert f(32, 16, 8, 4096, 128, 256) == 1
    # no small remainder over a multiple of the unit count: 160 pairs stay 160 workgroups (320
    # would leave 64 units a second workgroup each), 96 pairs become 480, 24 pairs 504
    assert f(20, 16, 8, 8192, 128, 256) == 1
    assert f(12, 16, 8, 16384, 128, 256) == 5
    assert f(3, 16, 8, 16384, 128, 256) == 21
    assert f(32, 16, 8, 8192, 128, 256) == 2


def test_static_scratch_entry_point_checks_its_limit_on_the_host(binding):
    lib = binding.load_library()
    static = lambda a: lib.parallax_decode_static(ctypes.byref(a), None)
    assert binding.parallax_decode_static_scratch_bytes() == 16384 * 260 * 4
    assert lib.parallax_decode_static(None, None) == binding.PLX_ERR_NULL
    a = _good_decode_args(binding); a.d = 96                  # the usual validation comes first
    assert static(a) == binding.PLX_ERR_SHAPE
    a = _good_decode_args(binding); a.B, a.Hq, a.Hkv, a.num_splits = 17, 8, 8, 128   # 17 408 records
    assert static(a) == binding.PLX_ERR_SCRATCH
    a = _good_decode_args(binding); a.B, a.Hq, a.Hkv, a.num_splits, a.Tq = 16, 8, 8, 128, 2
    assert static(a) == binding.PLX_ERR_SCRATCH
    assert "scratch" in binding.strerror(binding.PLX_ERR_SCRATCH)


def _good_decode_args(binding):
    a = binding.plx_decode_args()
    a.q = a.r = a.k = a.v = a.o = 0x1000
    a.B, a.Hq, a.Hkv, a.Lmax, a.d = 2, 4, 2, 64, 128
    a.k_stride_b, a.k_stride_h, a.k_stride_l = 2 * 64 * 128, 64 * 128, 128
    a.v_stride_b, a.v_stride_h, a.v_stride_l = 2 * 64 * 128, 64 * 128, 128
    a.scale, a.use_r, a.num_splits, a.dtype = 0.1, 1, 1, binding.PLX_BF16
    return a


def test_decode_rejects_bad_arguments_before_launch(binding):
    lib = binding.load_library()
    call = lambda a: lib.parallax_decode(ctypes.byref(a), None)
    assert lib.parallax_decode(None, None) == binding.PLX_ERR_NULL
    a = _good_decode_args(binding); a.k = None
    assert call(a) == binding.PLX_ERR_NULL
    a = _good_decode_args(binding); a.r = None
    assert call(a) == binding.PLX_ERR_NULL
    a = _good_decode_args(binding); a.Hq = 5
    assert call(a) == binding.PLX_ERR_SHAPE
    a = _good_decode_args(binding); a.d = 96
    assert call(a) == binding.PLX_ERR_SHAPE
    a = _good_decode_args(binding); a.Hq, a.Hkv = 34, 2      # G = 17 > 16
    assert call(a) == binding.PLX_ERR_SHAPE
    a = _good_decode_args(binding); a.Lmax = 0
    assert call(a) == binding.PLX_ERR_SHAPE
    a = _good_decode_args(binding); a.dtype = 7
    assert call(a) == binding.PLX_ERR_DTYPE
    a = _good_decode_args(binding); a.q = 0x1004
    assert call(a) == binding.PLX_ERR_ALIGN
    a = _good_decode_args(binding); a.k_stride_l = 132
    assert call(a) == binding.PLX_ERR_ALIGN
    a = _good_decode_args(binding); a.k_stride_l = 64
    assert call(a) == binding.PLX_ERR_SHAPE
    a = _good_decode_args(binding); a.num_splits = binding.PLX_MAX_SPLITS + 1
    assert call(a) == binding.PLX_ERR_SPLITS
    for bad in (-0.5, float("inf"), float("nan")):
        a = _good_decode_args(binding); a.scale = bad
        assert call(a) == binding.PLX_ERR_SCALE
    a = _good_decode_args(binding); a.num_splits = 4          # no workspace
    assert call(a) == binding.PLX_ERR_WORKSPACE
    a = _good_decode_args(binding); a.num_splits = 4
    a.workspace, a.workspace_bytes = 0x2000, 16
    assert call(a) == binding.PLX_ERR_WORKSPACE
    a = _good_decode_args(binding); a.window = -1
    assert call(a) == binding.PLX_ERR_SHAPE
    # in-kernel reduction: needs bf16, and workspace + counters as soon as there are splits
    fused = lib.parallax_decode_fused
    a = _good_decode_args(binding); a.num_splits = 4
    a.workspace, a.workspace_bytes = 0x2000, 1 << 30
    assert fused(ctypes.byref(a), None) == binding.PLX_ERR_WORKSPACE   # no counters
    a.split_counters = 0x4002
    assert fused(ctypes.byref(a), None) == binding.PLX_ERR_WORKSPACE   # misaligned counters
    a = _good_decode_args(binding); a.dtype = binding.PLX_F32
    assert fused(ctypes.byref(a), None) == binding.PLX_ERR_DTYPE
    # paged cache descriptors
    def paged():
        a = _good_decode_args(binding)
        a.block_table, a.page_size, a.block_table_stride, a.num_pages = 0x3000, 16, 4, 8
        return a
    a = paged(); a.block_table = 0x3002
    assert call(a) == binding.PLX_ERR_ALIGN
    a = paged(); a.page_size = 0
    assert call(a) == binding.PLX_ERR_SHAPE
    a = paged(); a.num_pages = 0
    assert call(a) == binding.PLX_ERR_SHAPE
    a = paged(); a.block_table_stride = 3                   # 3 pages x 16 rows < Lmax = 64
    assert call(a) == binding.PLX_ERR_SHAPE


def test_prefill_rejects_bad_arguments_before_launch(binding):
    lib = binding.load_library()

    def good():
        a = binding.plx_prefill_args()
        a.q = a.r = a.k = a.v = a.o = 0x1000
        a.B, a.Hq, a.Hkv, a.T, a.d = 1, 4, 2, 128, 128
        for name, H in (("q_stride", 4), ("r_stride", 4), ("o_stride", 4), ("k_stride", 2),
                        ("v_stride", 2)):
            setattr(a, name, (ctypes.c_int64 * 3)(H * 128 * 128, 128 * 128, 128))
        a.scale, a.causal, a.use_r, a.dtype = 0.1, 1, 1, binding.PLX_BF16
        return a

    call = lambda a: lib.parallax_prefill(ctypes.byref(a), None)
    assert lib.parallax_prefill(None, None) == binding.PLX_ERR_NULL
    a = good(); a.v = None
    assert call(a) == binding.PLX_ERR_NULL
    a = good(); a.Hkv = 3
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.d = 100
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.dtype = binding.PLX_F32; a.d = 260
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.o = 0x1008
    assert call(a) == binding.PLX_ERR_ALIGN
    a = good(); a.scale = -1.0
    assert call(a) == binding.PLX_ERR_SCALE
    a = good(); a.q_stride = (ctypes.c_int64 * 3)(4 * 128 * 128, 128 * 128, 130)
    assert call(a) == binding.PLX_ERR_ALIGN
    a = good(); a.k_stride = (ctypes.c_int64 * 3)(4 * 128 * 128, 128 * 128, 64)
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.Tkv = -1
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.Tkv = 64  # causal with fewer keys than query rows
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.window = -3
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.window, a.causal = 64, 0  # a window needs the rows' positions
    assert call(a) == binding.PLX_ERR_SHAPE
    # block-sparse lists: both arrays, shared or per batch / head, bf16 with the probe, no window
    def sparse():
        a = good()
        a.sparse_row_ptr, a.sparse_tile_idx, a.sparse_batch, a.sparse_heads = 0x5000, 0x6000, 1, 1
        return a
    a = sparse(); a.sparse_tile_idx = None
    assert call(a) == binding.PLX_ERR_NULL
    a = sparse(); a.sparse_heads = 3
    assert call(a) == binding.PLX_ERR_SHAPE
    a = sparse(); a.sparse_batch = 2
    assert call(a) == binding.PLX_ERR_SHAPE
    a = sparse(); a.window = 8
    assert call(a) == binding.PLX_ERR_SHAPE
    a = sparse(); a.use_r = 0
    assert call(a) == binding.PLX_ERR_SHAPE
    a = sparse(); a.sparse_row_ptr = 0x5002
    assert call(a) == binding.PLX_ERR_ALIGN


def test_util_argument_checks(binding):
    lib = binding.load_library()
    assert lib.parallax_util_copy(None, 0x1000, 16, None) == binding.PLX_ERR_NULL
    assert lib.parallax_util_copy(0x1000, 0x2000, 10, None) == binding.PLX_ERR_SHAPE
    assert lib.parallax_util_copy(0x1001, 0x2000, 16, None) == binding.PLX_ERR_ALIGN
    assert binding.parallax_util_read_sink_slots() > 0
    assert lib.parallax_util_mfma(256, 100, None, None) == binding.PLX_ERR_NULL
    assert lib.parallax_util_mfma(0, 100, 0x1000, None) == binding.PLX_ERR_SHAPE
    assert lib.parallax_util_mfma(256, 0, 0x1000, None) == binding.PLX_ERR_SHAPE
    assert lib.parallax_util_mfma(256, 100, 0x1002, None) == binding.PLX_ERR_ALIGN


def test_prefill_backward_rejects_bad_arguments_before_launch(binding):
    lib = binding.load_library()

    def good():
        a = binding.plx_prefill_bwd_args()
        for name in ("q", "r", "k", "v", "o", "vbar", "row_stats", "d_o", "dq", "dr", "dk", "dv"):
            setattr(a, name, 0x1000)
        a.B, a.Hq, a.Hkv, a.T, a.Tkv, a.d = 1, 4, 2, 128, 0, 128
        a.scale, a.causal, a.dtype = 0.1, 1, binding.PLX_BF16
        a.workspace, a.workspace_bytes = 0x2000, 1 * 4 * 128 * 16
        return a

    call = lambda a: lib.parallax_prefill_backward(ctypes.byref(a), None)
    assert binding.parallax_prefill_backward_workspace_bytes(1, 4, 128) == 4 * 128 * 16
    assert lib.parallax_prefill_backward(None, None) == binding.PLX_ERR_NULL
    a = good(); a.vbar = None
    assert call(a) == binding.PLX_ERR_NULL
    a = good(); a.dk = 0x1008
    assert call(a) == binding.PLX_ERR_ALIGN
    a = good(); a.dtype = 7
    assert call(a) == binding.PLX_ERR_DTYPE
    a = good(); a.d = 96
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.Tkv = 64
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.scale = float("nan")
    assert call(a) == binding.PLX_ERR_SCALE
    a = good(); a.workspace_bytes -= 1
    assert call(a) == binding.PLX_ERR_WORKSPACE
    a = good(); a.window = -1
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.window, a.causal = 16, 0     # a sliding window is causal
    assert call(a) == binding.PLX_ERR_SHAPE
    # the forward's row cache: both pointers or neither, with the probe
    f = binding.plx_prefill_args()
    f.q = f.r = f.k = f.v = f.o = 0x1000
    f.B, f.Hq, f.Hkv, f.T, f.d = 1, 4, 2, 128, 128
    for name, H in (("q_stride", 4), ("r_stride", 4), ("o_stride", 4), ("k_stride", 2), ("v_stride", 2)):
        setattr(f, name, (ctypes.c_int64 * 3)(H * 128 * 128, 128 * 128, 128))
    f.scale, f.causal, f.use_r, f.dtype = 0.1, 1, 1, binding.PLX_BF16
    f.vbar = 0x3000
    assert lib.parallax_prefill(ctypes.byref(f), None) == binding.PLX_ERR_NULL
    f.row_stats = 0x4000
    f.use_r = 0
    assert lib.parallax_prefill(ctypes.byref(f), None) == binding.PLX_ERR_SHAPE


def test_decode_mla_rejects_bad_arguments_before_launch(binding):
    lib = binding.load_library()

    def good():
        a = binding.plx_decode_mla_args()
        a.q = a.r = a.ckv = a.o = 0x1000
        a.B, a.Hq, a.Lmax, a.d_latent, a.d_rope, a.num_splits = 2, 16, 4096, 512, 64, 4
        a.ckv_stride_b, a.ckv_stride_l = 4096 * 576, 576
        a.scale, a.dtype = 0.05, binding.PLX_BF16
        a.workspace, a.workspace_bytes = 0x2000, binding.parallax_decode_mla_workspace_bytes(2, 16)
        return a

    call = lambda a: lib.parallax_decode_mla(ctypes.byref(a), None)
    assert binding.parallax_decode_mla_workspace_bytes(2, 16) == 2 * 16 * binding.PLX_MAX_SPLITS * 1028 * 4
    assert lib.parallax_decode_mla(None, None) == binding.PLX_ERR_NULL
    a = good(); a.ckv = None
    assert call(a) == binding.PLX_ERR_NULL
    a = good(); a.dtype = binding.PLX_F32
    assert call(a) == binding.PLX_ERR_DTYPE
    a = good(); a.d_latent, a.d_rope = 256, 64
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.ckv_stride_l = 512
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.ckv_stride_l = 580
    assert call(a) == binding.PLX_ERR_ALIGN
    a = good(); a.ckv_stride_l = (1 << 23) + 8
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.q = 0x1004
    assert call(a) == binding.PLX_ERR_ALIGN
    a = good(); a.scale = -1.0
    assert call(a) == binding.PLX_ERR_SCALE
    a = good(); a.num_splits = binding.PLX_MAX_SPLITS + 1
    assert call(a) == binding.PLX_ERR_SPLITS
    a = good(); a.workspace = None
    assert call(a) == binding.PLX_ERR_WORKSPACE
    a = good(); a.workspace_bytes = 100
    assert call(a) == binding.PLX_ERR_WORKSPACE
    a = good(); a.block_table, a.page_size, a.num_pages, a.block_table_stride = 0x3000, 64, 10, 8   # 512 < Lmax
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.block_table, a.page_size, a.num_pages, a.block_table_stride = 0x3000, 0, 10, 8
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.block_table, a.page_size, a.num_pages, a.block_table_stride = 0x3002, 64, 100, 64
    assert call(a) == binding.PLX_ERR_ALIGN
    # the split heuristic is host arithmetic with an explicit compute-unit count
    f = binding.parallax_decode_mla_num_splits
    assert f(64, 16, 16384, 256) == 4 and f(1, 16, 16384, 256) == 64 and f(1, 16, 100, 256) == 1
    assert f(512, 128, 4096, 256) == 1
    # more than 16 columns: 32 per workgroup, so 128 heads are four workgroups per (sequence, split)
    assert f(16, 128, 8192, 256) == 4 and f(64, 128, 4096, 256) == 1 and f(4, 128, 16384, 256) == 16
    assert f(24, 128, 8192, 256) == 5      # 96 x 5 = 480 workgroups: two rounds, the second nearly full
    for (B, Hq, L) in [(1, 1, 1), (3, 17, 5000), (128, 16, 131072), (2, 128, 70000)]:
        assert 1 <= f(B, Hq, L, 256) <= binding.PLX_MAX_SPLITS


def test_norm_rope_rejects_bad_arguments_before_launch(binding):
    lib = binding.load_library()

    def good():
        a = binding.plx_norm_rope_args()
        a.n_tensors, a.B, a.T, a.d = 2, 1, 4, 128
        for i in range(2):
            a.tensors[i].x = a.tensors[i].y = 0x1000
            a.tensors[i].gamma, a.tensors[i].H, a.tensors[i].rope = 0x2000, 2, 1
        a.eps, a.theta, a.dtype = 1e-6, 1.0e6, binding.PLX_BF16
        return a

    call = lambda a: lib.parallax_norm_rope(ctypes.byref(a), None)
    assert lib.parallax_norm_rope(None, None) == binding.PLX_ERR_NULL
    a = good(); a.n_tensors = 4
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.d = 96
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.dtype = binding.PLX_F32; a.d = 48
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.theta = 1.0
    assert call(a) == binding.PLX_ERR_SCALE
    a = good(); a.eps = float("nan")
    assert call(a) == binding.PLX_ERR_SCALE
    a = good(); a.tensors[1].gamma = None
    assert call(a) == binding.PLX_ERR_NULL
    a = good(); a.tensors[0].y = 0x1004
    assert call(a) == binding.PLX_ERR_ALIGN
    a = good(); a.tensors[1].H = 0
    assert call(a) == binding.PLX_ERR_SHAPE
    a = good(); a.pos0 = 0x3001
    assert call(a) == binding.PLX_ERR_ALIGN
    assert ctypes.sizeof(binding.plx_norm_rope_args) == 3 * 32 + 16 + 8 + 8 + 8 + 8 + 8


def test_block_mask_lists_by_rows_and_by_columns(binding):
    """The two list forms of a block mask (row blocks -> key tiles for the forward and the dQ / dR
    pass, key blocks of two tiles -> row blocks + flags for the dK / dV pass) against a
    brute-force reading of the mask."""
    import numpy as np
    import torch

    rng = np.random.default_rng(0)
    for shape in [(3, 5), (2, 3, 4, 7), (1, 4, 4, 8), (5, 1), (2, 6)]:
        bm = rng.random(shape) < 0.4
        if shape == (2, 6):
            bm[:] = False
        m = bm.reshape((1,) * (4 - bm.ndim) + bm.shape)
        Bs, Hs, nrb, nkt = m.shape
        row_ptr, tile_idx, gb, gh = binding.block_mask_lists(torch.as_tensor(bm))
        col_ptr, col_idx = binding.block_mask_column_lists(torch.as_tensor(bm))
        assert (gb, gh) == (Bs, Hs)
        assert len(row_ptr) == Bs * Hs * nrb + 1 and len(col_ptr) == Bs * Hs * ((nkt + 1) // 2) + 1
        e = 0
        for sb in range(Bs):
            for sh in range(Hs):
                for rb in range(nrb):
                    want = [t for t in range(nkt) if m[sb, sh, rb, t]]
                    assert tile_idx[row_ptr[e]:row_ptr[e + 1]].tolist() == want
                    e += 1
        e = 0
        for sb in range(Bs):
            for sh in range(Hs):
                for cb in range((nkt + 1) // 2):
                    want = []
                    for rb in range(nrb):
                        f = int(m[sb, sh, rb, 2 * cb]) + (2 * int(m[sb, sh, rb, 2 * cb + 1]) if 2 * cb + 1 < nkt else 0)
                        if f:
                            want.append(4 * rb + f)
                    assert col_idx[col_ptr[e]:col_ptr[e + 1]].tolist() == want
                    e += 1
