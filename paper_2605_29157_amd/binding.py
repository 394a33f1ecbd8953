"""Thin ctypes binding of the Parallax HIP library (same names as include/parallax.h).

Only argument marshalling happens here: torch tensors supply device pointers, strides and the
current HIP stream; every step of the attention path runs in the library's kernels. There is
no CPU or PyTorch fallback: if the library is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import os

import torch  # imported before the library so both share one HIP runtime

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libparallax_hip.so")

PLX_BF16, PLX_F32 = 0, 1
PLX_MAX_SPLITS = 128
(PLX_OK, PLX_ERR_NULL, PLX_ERR_SHAPE, PLX_ERR_DTYPE, PLX_ERR_ALIGN, PLX_ERR_WORKSPACE,
 PLX_ERR_LAUNCH, PLX_ERR_SPLITS, PLX_ERR_SCALE, PLX_ERR_SCRATCH) = (0, -1, -2, -3, -4, -5, -6, -7, -8, -9)
PLX_STATIC_SCRATCH_RECORDS = 16384

EXPORTED_SYMBOLS = (
    "parallax_decode_workspace_bytes", "parallax_decode_num_splits", "parallax_decode",
    "parallax_decode_partials", "parallax_decode_combine", "parallax_decode_fused",
    "parallax_decode_static", "parallax_decode_static_scratch_bytes",
    "parallax_decode_mla", "parallax_decode_mla_workspace_bytes", "parallax_decode_mla_num_splits",
    "parallax_prefill", "parallax_prefill_backward", "parallax_prefill_backward_workspace_bytes",
    "parallax_norm_rope", "parallax_rope_table", "parallax_util_copy", "parallax_util_read",
    "parallax_util_read_grid", "parallax_util_read_sink_slots", "parallax_util_mfma", "parallax_strerror", "parallax_version",
)


class plx_qr_prep(ctypes.Structure):
    _fields_ = [("q_gamma", ctypes.c_void_p), ("r_gamma", ctypes.c_void_p), ("rope_table", ctypes.c_void_p),
                ("pos0", ctypes.c_void_p), ("rope_positions", ctypes.c_int32), ("rope_q", ctypes.c_int32),
                ("rope_r", ctypes.c_int32), ("eps", ctypes.c_float)]


class plx_decode_args(ctypes.Structure):
    _fields_ = [
        ("q", ctypes.c_void_p), ("r", ctypes.c_void_p),
        ("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
        ("o", ctypes.c_void_p),
        ("seq_lens", ctypes.c_void_p),
        ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
        ("Lmax", ctypes.c_int32), ("d", ctypes.c_int32),
        ("k_stride_b", ctypes.c_int64), ("k_stride_h", ctypes.c_int64), ("k_stride_l", ctypes.c_int64),
        ("v_stride_b", ctypes.c_int64), ("v_stride_h", ctypes.c_int64), ("v_stride_l", ctypes.c_int64),
        ("scale", ctypes.c_float),
        ("use_r", ctypes.c_int32),
        ("num_splits", ctypes.c_int32),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("dtype", ctypes.c_int),
        ("block_table", ctypes.c_void_p),
        ("page_size", ctypes.c_int32), ("block_table_stride", ctypes.c_int32),
        ("num_pages", ctypes.c_int32),
        ("Tq", ctypes.c_int32),
        ("window", ctypes.c_int32),
        ("split_counters", ctypes.c_void_p),
        ("prep", plx_qr_prep),
    ]


class plx_prefill_args(ctypes.Structure):
    _fields_ = [
        ("q", ctypes.c_void_p), ("r", ctypes.c_void_p),
        ("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
        ("o", ctypes.c_void_p),
        ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
        ("T", ctypes.c_int32), ("d", ctypes.c_int32),
        ("q_stride", ctypes.c_int64 * 3), ("r_stride", ctypes.c_int64 * 3),
        ("k_stride", ctypes.c_int64 * 3), ("v_stride", ctypes.c_int64 * 3),
        ("o_stride", ctypes.c_int64 * 3),
        ("scale", ctypes.c_float),
        ("causal", ctypes.c_int32),
        ("use_r", ctypes.c_int32),
        ("dtype", ctypes.c_int),
        ("Tkv", ctypes.c_int32),
        ("window", ctypes.c_int32),
        ("vbar", ctypes.c_void_p), ("row_stats", ctypes.c_void_p),
        ("sparse_row_ptr", ctypes.c_void_p), ("sparse_tile_idx", ctypes.c_void_p),
        ("sparse_batch", ctypes.c_int32), ("sparse_heads", ctypes.c_int32),
        ("prep", plx_qr_prep),
    ]


class plx_prefill_bwd_args(ctypes.Structure):
    _fields_ = [
        ("q", ctypes.c_void_p), ("r", ctypes.c_void_p),
        ("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
        ("o", ctypes.c_void_p), ("vbar", ctypes.c_void_p),
        ("row_stats", ctypes.c_void_p),
        ("d_o", ctypes.c_void_p),
        ("dq", ctypes.c_void_p), ("dr", ctypes.c_void_p),
        ("dk", ctypes.c_void_p), ("dv", ctypes.c_void_p),
        ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
        ("T", ctypes.c_int32), ("Tkv", ctypes.c_int32), ("d", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("causal", ctypes.c_int32),
        ("dtype", ctypes.c_int), ("window", ctypes.c_int32),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("q_stride", ctypes.c_int64 * 3), ("r_stride", ctypes.c_int64 * 3), ("k_stride", ctypes.c_int64 * 3),
        ("v_stride", ctypes.c_int64 * 3), ("o_stride", ctypes.c_int64 * 3), ("vbar_stride", ctypes.c_int64 * 3),
        ("d_o_stride", ctypes.c_int64 * 3), ("dq_stride", ctypes.c_int64 * 3), ("dr_stride", ctypes.c_int64 * 3),
        ("dk_stride", ctypes.c_int64 * 3), ("dv_stride", ctypes.c_int64 * 3),
        ("sparse_row_ptr", ctypes.c_void_p), ("sparse_tile_idx", ctypes.c_void_p),
        ("sparse_col_ptr", ctypes.c_void_p), ("sparse_col_idx", ctypes.c_void_p),
        ("sparse_batch", ctypes.c_int32), ("sparse_heads", ctypes.c_int32),
    ]


class plx_decode_mla_args(ctypes.Structure):
    _fields_ = [
        ("q", ctypes.c_void_p), ("r", ctypes.c_void_p), ("ckv", ctypes.c_void_p), ("o", ctypes.c_void_p),
        ("seq_lens", ctypes.c_void_p),
        ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Lmax", ctypes.c_int32),
        ("d_latent", ctypes.c_int32), ("d_rope", ctypes.c_int32), ("num_splits", ctypes.c_int32),
        ("ckv_stride_b", ctypes.c_int64), ("ckv_stride_l", ctypes.c_int64),
        ("scale", ctypes.c_float), ("dtype", ctypes.c_int),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("block_table", ctypes.c_void_p),
        ("page_size", ctypes.c_int32), ("num_pages", ctypes.c_int32), ("block_table_stride", ctypes.c_int32),
        ("Tq", ctypes.c_int32), ("window", ctypes.c_int32),
    ]


class plx_norm_rope_tensor(ctypes.Structure):
    _fields_ = [("x", ctypes.c_void_p), ("y", ctypes.c_void_p), ("gamma", ctypes.c_void_p),
                ("H", ctypes.c_int32), ("rope", ctypes.c_int32)]


class plx_norm_rope_args(ctypes.Structure):
    _fields_ = [("tensors", plx_norm_rope_tensor * 3), ("n_tensors", ctypes.c_int32),
                ("B", ctypes.c_int32), ("T", ctypes.c_int32), ("d", ctypes.c_int32),
                ("pos0", ctypes.c_void_p), ("eps", ctypes.c_float), ("theta", ctypes.c_float),
                ("dtype", ctypes.c_int), ("rope_table", ctypes.c_void_p), ("table_positions", ctypes.c_int32)]


class ParallaxError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (status %d)" % (where, strerror(status), status))


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libparallax_hip.so (built by __graft_entry__.build()). Raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "%s is missing: build it with `python -c 'import __graft_entry__ as g; "
                "g.build()'` (there is no fallback path)" % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        lib.parallax_decode_workspace_bytes.argtypes = [ctypes.c_int32] * 5
        lib.parallax_decode_workspace_bytes.restype = ctypes.c_size_t
        lib.parallax_decode_num_splits.argtypes = [ctypes.c_int32] * 6
        lib.parallax_decode_num_splits.restype = ctypes.c_int32
        lib.parallax_decode.argtypes = [ctypes.POINTER(plx_decode_args), ctypes.c_void_p]
        lib.parallax_decode.restype = ctypes.c_int
        lib.parallax_decode_static_scratch_bytes.argtypes = []
        lib.parallax_decode_static_scratch_bytes.restype = ctypes.c_size_t
        for name in ("parallax_decode_partials", "parallax_decode_combine", "parallax_decode_fused",
                     "parallax_decode_static"):
            getattr(lib, name).argtypes = [ctypes.POINTER(plx_decode_args), ctypes.c_void_p]
            getattr(lib, name).restype = ctypes.c_int
        lib.parallax_prefill.argtypes = [ctypes.POINTER(plx_prefill_args), ctypes.c_void_p]
        lib.parallax_prefill.restype = ctypes.c_int
        lib.parallax_prefill_backward.argtypes = [ctypes.POINTER(plx_prefill_bwd_args), ctypes.c_void_p]
        lib.parallax_prefill_backward.restype = ctypes.c_int
        lib.parallax_prefill_backward_workspace_bytes.argtypes = [ctypes.c_int32] * 3
        lib.parallax_prefill_backward_workspace_bytes.restype = ctypes.c_size_t
        lib.parallax_norm_rope.argtypes = [ctypes.POINTER(plx_norm_rope_args), ctypes.c_void_p]
        lib.parallax_norm_rope.restype = ctypes.c_int
        lib.parallax_rope_table.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_float,
                                            ctypes.c_void_p]
        lib.parallax_rope_table.restype = ctypes.c_int
        lib.parallax_util_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                           ctypes.c_void_p]
        lib.parallax_util_copy.restype = ctypes.c_int
        lib.parallax_util_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                           ctypes.c_void_p]
        lib.parallax_util_read.restype = ctypes.c_int
        lib.parallax_util_read_grid.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int32,
                                                ctypes.c_void_p]
        lib.parallax_util_read_grid.restype = ctypes.c_int
        lib.parallax_decode_mla.argtypes = [ctypes.POINTER(plx_decode_mla_args), ctypes.c_void_p]
        lib.parallax_decode_mla.restype = ctypes.c_int
        lib.parallax_decode_mla_workspace_bytes.argtypes = [ctypes.c_int32] * 2
        lib.parallax_decode_mla_workspace_bytes.restype = ctypes.c_size_t
        lib.parallax_decode_mla_num_splits.argtypes = [ctypes.c_int32] * 4
        lib.parallax_decode_mla_num_splits.restype = ctypes.c_int32
        lib.parallax_util_mfma.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
        lib.parallax_util_mfma.restype = ctypes.c_int
        lib.parallax_util_read_sink_slots.argtypes = []
        lib.parallax_util_read_sink_slots.restype = ctypes.c_int32
        lib.parallax_strerror.argtypes = [ctypes.c_int]
        lib.parallax_strerror.restype = ctypes.c_char_p
        lib.parallax_version.argtypes = []
        lib.parallax_version.restype = ctypes.c_int
        _lib = lib
    return _lib


def strerror(status: int) -> str:
    return load_library().parallax_strerror(int(status)).decode()


def version() -> int:
    return int(load_library().parallax_version())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return PLX_BF16
    if t.dtype == torch.float32:
        return PLX_F32
    raise TypeError("Parallax kernels take bfloat16 or float32 tensors, got %s" % t.dtype)


def _stream_ptr(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def parallax_rope_table(n_pos, d, theta=1.0e6, device="cuda:0", stream=None):
    """(cos, sin) of pos * theta^(-2i/d): fp32 tensor [n_pos, d/2, 2] for qr_prep()."""
    table = torch.empty(n_pos, d // 2, 2, dtype=torch.float32, device=device)
    st = load_library().parallax_rope_table(table.data_ptr(), int(n_pos), int(d), float(theta), _stream_ptr(stream))
    if st != PLX_OK:
        raise ParallaxError(st, "parallax_rope_table")
    return table


def qr_prep(q_gamma, r_gamma, rope_table=None, pos0=None, rope_q=True, rope_r=True, eps=1e-6):
    """Fill a plx_qr_prep (RMSNorm + RoPE on q, rho inside the attention kernels) from tensors. The
    returned struct only holds pointers: keep the tensors alive until the call has been enqueued."""
    a = plx_qr_prep()
    for g in (q_gamma, r_gamma):
        if g is not None and (g.dtype != torch.float32 or not g.is_cuda or not g.is_contiguous()):
            raise TypeError("RMSNorm weights must be contiguous fp32 device tensors")
    a.q_gamma = q_gamma.data_ptr()
    a.r_gamma = r_gamma.data_ptr() if r_gamma is not None else None
    if rope_table is not None:
        if rope_table.dtype != torch.float32 or not rope_table.is_contiguous():
            raise TypeError("rope_table must be a contiguous fp32 tensor [n_pos, d/2, 2]")
        a.rope_table, a.rope_positions = rope_table.data_ptr(), rope_table.shape[0]
        a.rope_q, a.rope_r = (1 if rope_q else 0), (1 if rope_r else 0)
    if pos0 is not None:
        if pos0.dtype != torch.int32:
            raise TypeError("pos0 must be int32")
        a.pos0 = pos0.data_ptr()
    a.eps = float(eps)
    return a


def parallax_decode_workspace_bytes(B, Hq, Hkv, Lmax, d) -> int:
    return int(load_library().parallax_decode_workspace_bytes(B, Hq, Hkv, Lmax, d))


def parallax_decode_num_splits(B, Hq, Hkv, Lmax, d, num_cus=0) -> int:
    return int(load_library().parallax_decode_num_splits(B, Hq, Hkv, Lmax, d, num_cus))


def decode_args(q, r, k, v, out, scale, seq_lens=None, use_r=True, num_splits=0, workspace=None,
                block_table=None, max_len=None, window=0):
    """Fill a plx_decode_args from tensors: q, r, out [B, Hq, d]; k, v [B, Hkv, Lmax, d], or,
    with block_table [B, pages per sequence] (int32), page pools [num_pages, Hkv, page_size, d]
    (max_len = largest logical length, default: pages per sequence x page_size).
    q, r, out may also be [B, Hq, Tq, d]: Tq query rows, the last Tq positions of each sequence."""
    Tq = 1
    if q.dim() == 4:
        Tq = q.shape[2]
    B, Hq, d = q.shape[0], q.shape[1], q.shape[-1]
    _, Hkv, Lmax, _ = k.shape
    if block_table is not None:
        Lmax = int(max_len) if max_len is not None else block_table.shape[1] * k.shape[2]
    a = plx_decode_args()
    a.q, a.k, a.v, a.o = q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr()
    a.r = r.data_ptr() if r is not None else None
    a.seq_lens = seq_lens.data_ptr() if seq_lens is not None else None
    a.B, a.Hq, a.Hkv, a.Lmax, a.d = B, Hq, Hkv, Lmax, d
    a.k_stride_b, a.k_stride_h, a.k_stride_l = k.stride(0), k.stride(1), k.stride(2)
    a.v_stride_b, a.v_stride_h, a.v_stride_l = v.stride(0), v.stride(1), v.stride(2)
    a.scale = float(scale)
    a.use_r = 1 if use_r else 0
    a.num_splits = int(num_splits)
    if workspace is not None:
        a.workspace = workspace.data_ptr()
        a.workspace_bytes = workspace.numel() * workspace.element_size()
    a.dtype = _dtype_code(q)
    a.Tq = Tq
    a.window = int(window)
    if block_table is not None:
        a.block_table = block_table.data_ptr()
        a.page_size, a.block_table_stride, a.num_pages = k.shape[2], block_table.stride(0), k.shape[0]
    return a


def parallax_decode(q, r, k, v, scale, seq_lens=None, use_r=True, num_splits=0, workspace=None,
                    out=None, stream=None, block_table=None, max_len=None, split_counters=None,
                    window=0, prep=None):
    """Single-step Parallax decode. Allocates `out` / `workspace` with torch when not given
    (allocation only; all arithmetic is in the library). With `split_counters` (zeroed int32
    device tensor, >= B * Hkv entries) the call goes to parallax_decode_fused: one launch, the
    last split of every group to arrive merges inside the kernel."""
    for t in (q, k, v) + ((r,) if r is not None else ()):
        if not t.is_cuda:
            raise ValueError("parallax_decode needs device tensors")
    if q.stride(-1) != 1 or k.stride(-1) != 1 or v.stride(-1) != 1 or not q.is_contiguous() or (
            r is not None and not r.is_contiguous()):
        raise ValueError("q, r must be contiguous and k, v contiguous in the last dimension")
    if seq_lens is not None and seq_lens.dtype != torch.int32:
        raise TypeError("seq_lens must be int32")
    B, Hq, d = q.shape[0], q.shape[1], q.shape[-1]
    Tq = q.shape[2] if q.dim() == 4 else 1
    _, Hkv, Lmax, _ = k.shape
    if block_table is not None:
        if block_table.dtype != torch.int32 or not block_table.is_cuda or block_table.stride(1) != 1:
            raise TypeError("block_table must be an int32 device tensor [B, pages per sequence]")
        if block_table.shape[0] != B or v.shape != k.shape:
            raise ValueError("block_table needs one row per sequence; k and v pools of one shape")
        Lmax = int(max_len) if max_len is not None else block_table.shape[1] * k.shape[2]
    if out is None:
        out = torch.empty_like(q)
    if workspace is None and num_splits != 1 and q.dtype == torch.bfloat16:
        # (with a window the library may pick fewer splits than for Lmax, never more)
        S = num_splits or parallax_decode_num_splits(B, Hq, Hkv, Lmax, d)
        if S > 1:
            workspace = torch.empty(B * Hq * Tq * S * (2 * d + 4), dtype=torch.float32,
                                    device=q.device)
    a = decode_args(q, r, k, v, out, scale, seq_lens, use_r, num_splits, workspace, block_table,
                    max_len, window)
    if prep is not None:
        a.prep = prep
    entry = "parallax_decode"
    if split_counters is not None:
        if (split_counters.dtype != torch.int32 or not split_counters.is_cuda
                or not split_counters.is_contiguous() or split_counters.numel() < B * Hkv):
            raise TypeError("split_counters must be a contiguous int32 device tensor, >= B * Hkv")
        a.split_counters = split_counters.data_ptr()
        entry = "parallax_decode_fused"
    st = getattr(load_library(), entry)(ctypes.byref(a), _stream_ptr(stream))
    if st != PLX_OK:
        raise ParallaxError(st, entry)
    return out


def parallax_decode_static_scratch_bytes() -> int:
    return int(load_library().parallax_decode_static_scratch_bytes())


def parallax_decode_static(q, r, k, v, scale, out, seq_lens=None, use_r=True, num_splits=0,
                           stream=None, block_table=None, max_len=None, window=0):
    """parallax_decode with the split records in the library's own fixed scratch: nothing is
    allocated here or in the library; `out` is the caller's."""
    a = decode_args(q, r, k, v, out, scale, seq_lens, use_r, num_splits, None, block_table, max_len,
                    window)
    st = load_library().parallax_decode_static(ctypes.byref(a), _stream_ptr(stream))
    if st != PLX_OK:
        raise ParallaxError(st, "parallax_decode_static")
    return out


def parallax_decode_fused(q, r, k, v, scale, split_counters, **kw):
    """parallax_decode with the merge inside the split kernel; see parallax_decode."""
    return parallax_decode(q, r, k, v, scale, split_counters=split_counters, **kw)


def parallax_decode_partials(q, r, k, v, scale, num_splits, workspace, seq_lens=None, use_r=True,
                             stream=None):
    """Split kernel only: fills `workspace` with the (m, d1, d2, pad, O1, O2) records."""
    a = decode_args(q, r, k, v, q, scale, seq_lens, use_r, num_splits, workspace)
    a.o = None
    st = load_library().parallax_decode_partials(ctypes.byref(a), _stream_ptr(stream))
    if st != PLX_OK:
        raise ParallaxError(st, "parallax_decode_partials")
    return workspace


def parallax_decode_combine(workspace, out, Hkv, num_splits, stream=None):
    """Merge kernel only: `workspace` holds num_splits records per (b, hq); writes out [B, Hq, d]."""
    B, Hq, d = out.shape
    a = plx_decode_args()
    a.o = out.data_ptr()
    a.B, a.Hq, a.Hkv, a.Lmax, a.d = B, Hq, Hkv, 1, d
    a.num_splits = int(num_splits)
    a.workspace = workspace.data_ptr()
    a.workspace_bytes = workspace.numel() * workspace.element_size()
    a.dtype = _dtype_code(out)
    st = load_library().parallax_decode_combine(ctypes.byref(a), _stream_ptr(stream))
    if st != PLX_OK:
        raise ParallaxError(st, "parallax_decode_combine")
    return out


def prefill_args(q, r, k, v, out, scale, causal=True, use_r=True, window=0):
    """Fill a plx_prefill_args from tensors: q, r, out [B, Hq, T, d]; k, v [B, Hkv, Tkv, d]."""
    B, Hq, T, d = q.shape
    Hkv, Tkv = k.shape[1], k.shape[2]
    a = plx_prefill_args()
    a.q, a.k, a.v, a.o = q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr()
    a.r = r.data_ptr() if r is not None else None
    a.B, a.Hq, a.Hkv, a.T, a.d = B, Hq, Hkv, T, d
    for name, t in (("q_stride", q), ("r_stride", r if r is not None else q), ("k_stride", k),
                    ("v_stride", v), ("o_stride", out)):
        setattr(a, name, (ctypes.c_int64 * 3)(t.stride(0), t.stride(1), t.stride(2)))
    a.scale = float(scale)
    a.causal = 1 if causal else 0
    a.use_r = 1 if use_r else 0
    a.dtype = _dtype_code(q)
    a.Tkv = Tkv
    a.window = int(window)
    return a


BLOCK_ROWS, BLOCK_KEYS = 128, 64  # the block-sparse granularity: the prefill kernel's tiles


def block_mask_lists(block_mask):
    """Block mask [(B,) (Hq,) ceil(T/128), ceil(Tkv/64)] (bool, device) -> (row_ptr, tile_idx,
    sparse_batch, sparse_heads) for plx_prefill_args: per row block the ascending indices of its
    key tiles. Index bookkeeping only."""
    m = block_mask.to(torch.bool)
    while m.dim() < 4:
        m = m.unsqueeze(0)
    Bs, Hs, nrb, nkt = m.shape
    flat = m.reshape(-1, nkt)
    counts = flat.sum(dim=1)
    row_ptr = torch.zeros(flat.shape[0] + 1, dtype=torch.int32, device=m.device)
    row_ptr[1:] = torch.cumsum(counts, 0).to(torch.int32)
    tile_idx = torch.nonzero(flat)[:, 1].to(torch.int32).contiguous()  # row-major: ascending per row
    if tile_idx.numel() == 0:
        tile_idx = torch.zeros(1, dtype=torch.int32, device=m.device)
    return row_ptr, tile_idx, Bs, Hs


def block_mask_column_lists(block_mask):
    """The same cells by columns, for plx_prefill_bwd_args: per key block of 128 keys (two key
    tiles) the ascending row blocks that list one of its tiles, each entry 4 * row block + flags
    (flag bit t: key tile 2 * cb + t is listed). Returns (col_ptr, col_idx). Index bookkeeping only."""
    m = block_mask.to(torch.bool)
    while m.dim() < 4:
        m = m.unsqueeze(0)
    Bs, Hs, nrb, nkt = m.shape
    if nkt % 2:
        m = torch.cat([m, torch.zeros(Bs, Hs, nrb, 1, dtype=torch.bool, device=m.device)], dim=-1)
    pair = m.reshape(Bs, Hs, nrb, -1, 2)                      # [.., rb, cb, t]
    flags = pair[..., 0].to(torch.int32) + 2 * pair[..., 1].to(torch.int32)
    by_col = flags.transpose(-1, -2).reshape(-1, nrb)         # one line per (sb, sh, cb)
    hit = by_col > 0
    col_ptr = torch.zeros(by_col.shape[0] + 1, dtype=torch.int32, device=m.device)
    col_ptr[1:] = torch.cumsum(hit.sum(dim=1), 0).to(torch.int32)
    where = torch.nonzero(hit)                                # row-major: ascending row blocks per line
    col_idx = (4 * where[:, 1].to(torch.int32) + by_col[hit]).to(torch.int32).contiguous()
    if col_idx.numel() == 0:
        col_idx = torch.zeros(1, dtype=torch.int32, device=m.device)
    return col_ptr, col_idx


def parallax_prefill(q, r, k, v, scale, causal=True, use_r=True, out=None, stream=None, window=0,
                     save_for_backward=False, block_mask=None, prep=None):
    """Parallax prefill forward over T query rows and Tkv keys (causal: the rows are the last
    T positions of the Tkv-long sequence). With save_for_backward the kernel also writes the row
    cache of the backward pass and (out, vbar, row_stats) is returned."""
    for t in (q, k, v) + ((r,) if r is not None else ()):
        if not t.is_cuda:
            raise ValueError("parallax_prefill needs device tensors")
        if t.stride(-1) != 1:
            raise ValueError("the last dimension must be contiguous")
    if v.shape[2] != k.shape[2]:
        raise ValueError("k and v must hold the same number of keys")
    if out is None:
        out = torch.empty_like(q)
    a = prefill_args(q, r, k, v, out, scale, causal, use_r, window)
    if block_mask is not None:
        nrb, nkt = -(-q.shape[2] // BLOCK_ROWS), -(-k.shape[2] // BLOCK_KEYS)
        if tuple(block_mask.shape[-2:]) != (nrb, nkt):
            raise ValueError("block_mask must end in [ceil(T/128), ceil(Tkv/64)] = [%d, %d]" % (nrb, nkt))
        row_ptr, tile_idx, Bs, Hs = block_mask_lists(block_mask.to(q.device))
        a.sparse_row_ptr, a.sparse_tile_idx = row_ptr.data_ptr(), tile_idx.data_ptr()
        a.sparse_batch, a.sparse_heads = Bs, Hs
    if prep is not None:
        a.prep = prep
    if save_for_backward:
        vbar = torch.empty_like(out)
        row_stats = torch.empty(q.shape[:3] + (2,), dtype=torch.float32, device=q.device)
        a.vbar, a.row_stats = vbar.data_ptr(), row_stats.data_ptr()
    st = load_library().parallax_prefill(ctypes.byref(a), _stream_ptr(stream))
    if st != PLX_OK:
        raise ParallaxError(st, "parallax_prefill")
    return (out, vbar, row_stats) if save_for_backward else out


def parallax_prefill_backward_workspace_bytes(B, Hq, T) -> int:
    return int(load_library().parallax_prefill_backward_workspace_bytes(B, Hq, T))


def prefill_bwd_args(q, r, k, v, o, vbar, row_stats, d_o, dq, dr, dk, dv, scale, causal, workspace, window=0):
    """Fill a plx_prefill_bwd_args: [B, H, T, d] tensors (views with any batch / head / row strides,
    last dimension contiguous); row_stats and the workspace dense."""
    for t in (q, r, k, v, o, vbar, row_stats, d_o, dq, dr, dk, dv, workspace):
        if not t.is_cuda or t.stride(-1) != 1:
            raise ValueError("parallax_prefill_backward needs device tensors with a contiguous last dimension")
    if not row_stats.is_contiguous() or not workspace.is_contiguous():
        raise ValueError("row_stats and the workspace must be contiguous")
    B, Hq, T, d = q.shape
    a = plx_prefill_bwd_args()
    a.q, a.r, a.k, a.v = q.data_ptr(), r.data_ptr(), k.data_ptr(), v.data_ptr()
    a.o, a.vbar, a.row_stats, a.d_o = o.data_ptr(), vbar.data_ptr(), row_stats.data_ptr(), d_o.data_ptr()
    a.dq, a.dr, a.dk, a.dv = dq.data_ptr(), dr.data_ptr(), dk.data_ptr(), dv.data_ptr()
    a.B, a.Hq, a.Hkv, a.T, a.Tkv, a.d = B, Hq, k.shape[1], T, k.shape[2], d
    a.scale = float(scale)
    a.causal = 1 if causal else 0
    a.window = int(window)
    a.dtype = _dtype_code(q)
    a.workspace = workspace.data_ptr()
    a.workspace_bytes = workspace.numel() * workspace.element_size()
    for name, t in (("q", q), ("r", r), ("k", k), ("v", v), ("o", o), ("vbar", vbar), ("d_o", d_o),
                    ("dq", dq), ("dr", dr), ("dk", dk), ("dv", dv)):
        setattr(a, name + "_stride", (ctypes.c_int64 * 3)(*t.stride()[:3]))
    return a


def parallax_prefill_backward(q, r, k, v, o, vbar, row_stats, d_o, scale, causal=True, stream=None,
                              workspace=None, window=0, block_mask=None):
    """Gradients (dq, dr, dk, dv) of parallax_prefill for the upstream gradient d_o, from the
    forward's output and row cache (save_for_backward=True, same causal / window / block_mask)."""
    dq, dr = torch.empty_like(q), torch.empty_like(q)
    dk, dv = torch.empty_like(k), torch.empty_like(k)
    if workspace is None:
        workspace = torch.empty(q.shape[0] * q.shape[1] * q.shape[2] * 4, dtype=torch.float32,
                                device=q.device)
    a = prefill_bwd_args(q, r, k, v, o, vbar, row_stats, d_o, dq, dr, dk, dv, scale, causal, workspace, window)
    if block_mask is not None:
        nrb, nkt = -(-q.shape[2] // BLOCK_ROWS), -(-k.shape[2] // BLOCK_KEYS)
        if tuple(block_mask.shape[-2:]) != (nrb, nkt):
            raise ValueError("block_mask must end in [ceil(T/128), ceil(Tkv/64)] = [%d, %d]" % (nrb, nkt))
        row_ptr, tile_idx, Bs, Hs = block_mask_lists(block_mask.to(q.device))
        col_ptr, col_idx = block_mask_column_lists(block_mask.to(q.device))
        a.sparse_row_ptr, a.sparse_tile_idx = row_ptr.data_ptr(), tile_idx.data_ptr()
        a.sparse_col_ptr, a.sparse_col_idx = col_ptr.data_ptr(), col_idx.data_ptr()
        a.sparse_batch, a.sparse_heads = Bs, Hs
    st = load_library().parallax_prefill_backward(ctypes.byref(a), _stream_ptr(stream))
    if st != PLX_OK:
        raise ParallaxError(st, "parallax_prefill_backward")
    return dq, dr, dk, dv


def norm_rope_args(tensors, pos0=None, eps=1e-6, theta=1.0e6, rope_table=None):
    """Fill a plx_norm_rope_args. tensors: up to three (x, gamma, rope, out) with x, out
    [B, H, T, d] contiguous (out may be x) and gamma [d] fp32."""
    a = plx_norm_rope_args()
    a.n_tensors = len(tensors)
    B, _, T, d = tensors[0][0].shape
    for i, (x, gamma, use_rope, out) in enumerate(tensors):
        if not (x.is_cuda and x.is_contiguous() and out.is_contiguous() and gamma.dtype == torch.float32):
            raise ValueError("parallax_norm_rope needs contiguous device tensors and fp32 weights")
        if x.shape[0] != B or x.shape[2] != T or x.shape[3] != d or out.shape != x.shape:
            raise ValueError("the tensors of one call share B, T and d")
        a.tensors[i].x, a.tensors[i].y, a.tensors[i].gamma = x.data_ptr(), out.data_ptr(), gamma.data_ptr()
        a.tensors[i].H, a.tensors[i].rope = x.shape[1], 1 if use_rope else 0
    a.B, a.T, a.d = B, T, d
    a.pos0 = pos0.data_ptr() if pos0 is not None else None
    a.eps, a.theta = float(eps), float(theta)
    a.dtype = _dtype_code(tensors[0][0])
    if rope_table is not None:  # [n_pos, d / 2, 2] fp32 from parallax_rope_table (same d, theta)
        if rope_table.dtype != torch.float32 or not rope_table.is_contiguous() or rope_table.shape[1] != d // 2:
            raise ValueError("rope_table must be the contiguous fp32 [n_pos, d/2, 2] table of this d")
        a.rope_table, a.table_positions = rope_table.data_ptr(), rope_table.shape[0]
    return a


def parallax_norm_rope(tensors, pos0=None, eps=1e-6, theta=1.0e6, stream=None, inplace=False, rope_table=None):
    """RMSNorm + RoPE on up to three tensors in one launch. tensors: list of (x, gamma, rope);
    returns the list of results (the inputs themselves with inplace=True)."""
    if pos0 is not None and pos0.dtype != torch.int32:
        raise TypeError("pos0 must be int32")
    full = [(x, g, rp, x if inplace else torch.empty_like(x)) for (x, g, rp) in tensors]
    a = norm_rope_args(full, pos0, eps, theta, rope_table)
    st = load_library().parallax_norm_rope(ctypes.byref(a), _stream_ptr(stream))
    if st != PLX_OK:
        raise ParallaxError(st, "parallax_norm_rope")
    return [t[3] for t in full]


def parallax_decode_mla_workspace_bytes(B, Hq) -> int:
    return int(load_library().parallax_decode_mla_workspace_bytes(B, Hq))


def parallax_decode_mla_num_splits(B, Hq, Lmax, num_cus=0) -> int:
    return int(load_library().parallax_decode_mla_num_splits(B, Hq, Lmax, num_cus))


def decode_mla_args(q, r, ckv, out, scale, seq_lens=None, num_splits=0, workspace=None, d_latent=512,
                    block_table=None, max_len=None, window=0):
    """Fill a plx_decode_mla_args: q, r [B, Hq, dk] and out [B, Hq, d_latent] contiguous (or, with
    several query rows per head at the last positions of the sequence, [B, Hq, Tq, dk] and
    [B, Hq, Tq, d_latent]), ckv [B, L, dk] with any batch / token strides -- or, with an int32
    block_table [B, pages], a page pool [num_pages, page_size, dk] (max_len = capacity in tokens,
    default pages * page_size)."""
    for t in (q, r, out):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("parallax_decode_mla needs contiguous device tensors for q, r and out")
    if not ckv.is_cuda or ckv.stride(-1) != 1:
        raise ValueError("the last dimension of the cache must be contiguous")
    a = plx_decode_mla_args()
    a.q, a.r, a.ckv, a.o = q.data_ptr(), r.data_ptr(), ckv.data_ptr(), out.data_ptr()
    a.seq_lens = seq_lens.data_ptr() if seq_lens is not None else None
    a.B, a.Hq, a.Lmax = q.shape[0], q.shape[1], ckv.shape[1]
    if block_table is not None:
        if block_table.dtype != torch.int32 or not block_table.is_cuda or block_table.stride(-1) != 1:
            raise ValueError("block_table must be a device int32 tensor with a contiguous last dimension")
        a.block_table = block_table.data_ptr()
        a.page_size, a.num_pages, a.block_table_stride = ckv.shape[1], ckv.shape[0], block_table.stride(0)
        a.Lmax = int(max_len) if max_len is not None else block_table.shape[1] * ckv.shape[1]
    a.d_latent, a.d_rope = d_latent, q.shape[-1] - d_latent
    a.Tq = q.shape[2] if q.dim() == 4 else 1
    a.window = int(window)
    a.num_splits = int(num_splits)
    a.ckv_stride_b, a.ckv_stride_l = ckv.stride(0), ckv.stride(1)
    a.scale = float(scale)
    a.dtype = _dtype_code(q)
    if workspace is not None:
        a.workspace = workspace.data_ptr()
        a.workspace_bytes = workspace.numel() * workspace.element_size()
    return a


def parallax_decode_mla(q, r, ckv, scale, seq_lens=None, num_splits=0, out=None, workspace=None,
                        stream=None, d_latent=512, block_table=None, max_len=None, window=0):
    """Parallax attention over an MLA-style latent cache: key = the whole cached row, value = its
    first d_latent numbers, shared by all heads. q, r [B, Hq, dk] (one decode row) or
    [B, Hq, Tq, dk] (rows at the last Tq positions, causal among themselves: a chunked decode
    step, or the prefill over the latent cache with Tq = prompt length); window > 0 = sliding."""
    if out is None:
        out = torch.empty(q.shape[:-1] + (d_latent,), dtype=q.dtype, device=q.device)
    n_cols = q.shape[1] * (q.shape[2] if q.dim() == 4 else 1)
    if workspace is None and num_splits != 1:
        lmax = ckv.shape[1] if block_table is None else (
            int(max_len) if max_len is not None else block_table.shape[1] * ckv.shape[1])
        S = num_splits or parallax_decode_mla_num_splits(q.shape[0], n_cols, lmax)
        if S > 1:
            workspace = torch.empty(q.shape[0] * n_cols * S * (2 * d_latent + 4), dtype=torch.float32,
                                    device=q.device)
    a = decode_mla_args(q, r, ckv, out, scale, seq_lens, num_splits, workspace, d_latent, block_table, max_len,
                        window)
    st = load_library().parallax_decode_mla(ctypes.byref(a), _stream_ptr(stream))
    if st != PLX_OK:
        raise ParallaxError(st, "parallax_decode_mla")
    return out


def parallax_util_copy(dst, src, stream=None):
    nbytes = src.numel() * src.element_size()
    st = load_library().parallax_util_copy(dst.data_ptr(), src.data_ptr(), nbytes,
                                           _stream_ptr(stream))
    if st != PLX_OK:
        raise ParallaxError(st, "parallax_util_copy")
    return dst


def parallax_util_read(src, sink, stream=None):
    nbytes = src.numel() * src.element_size()
    st = load_library().parallax_util_read(src.data_ptr(), nbytes, sink.data_ptr(),
                                           _stream_ptr(stream))
    if st != PLX_OK:
        raise ParallaxError(st, "parallax_util_read")
    return sink


def parallax_util_read_grid(src, sink, workgroups, nbytes=None, stream=None):
    """Plain read of the first nbytes of src (default: all of it) by `workgroups` workgroups."""
    if nbytes is None:
        nbytes = src.numel() * src.element_size()
    st = load_library().parallax_util_read_grid(src.data_ptr(), int(nbytes), sink.data_ptr(), int(workgroups),
                                                _stream_ptr(stream))
    if st != PLX_OK:
        raise ParallaxError(st, "parallax_util_read_grid")
    return sink


def parallax_util_mfma(workgroups, iters, sink, stream=None) -> float:
    """Register-only bf16 MFMA loop; returns the flops it performs. sink: >= workgroups * 1024 bytes."""
    if sink.numel() * sink.element_size() < workgroups * 1024:
        raise ValueError("sink too small")
    st = load_library().parallax_util_mfma(int(workgroups), int(iters), sink.data_ptr(), _stream_ptr(stream))
    if st != PLX_OK:
        raise ParallaxError(st, "parallax_util_mfma")
    return float(workgroups) * 4 * iters * 8 * 32768


def parallax_util_read_sink_slots() -> int:
    return int(load_library().parallax_util_read_sink_slots())
