"""ctypes front end of the C double-precision Parallax oracle (test infrastructure).

The arithmetic lives in ``parallax_oracle.c`` (the paper's forward equation, Sec. 3.1,
in its re-weighted softmax form). This file only builds that C file with gcc, loads it
and marshals numpy arrays. Nothing here is imported by the product package; only the
tests, the smoke check and the benchmark's ``cpu_baseline`` leg use it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "parallax_oracle.c")
_LIB = os.path.join(_HERE, "libparallax_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2 -fopenmp). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _bind(path):
    """Load an oracle library (the built one, or a mutant a test compiled) and type it."""
    lib = ctypes.CDLL(path)
    common = [ctypes.c_int] * 6 + [ctypes.c_double, ctypes.c_int, ctypes.c_void_p,
                                   ctypes.c_void_p, ctypes.c_int64, ctypes.c_int]
    lib.plx_oracle_f64.argtypes = [ctypes.c_void_p] * 5 + common
    lib.plx_oracle_f64.restype = ctypes.c_int
    lib.plx_oracle_f32in.argtypes = [ctypes.c_void_p] * 5 + common
    lib.plx_oracle_f32in.restype = ctypes.c_int
    lib.plx_oracle_num_threads.restype = ctypes.c_int
    return lib


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = _bind(_LIB)
    return _lib


def num_threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    return int(_load().plx_oracle_num_threads())


def forward(q, r, k, v, scale, causal=False, seq_lens=None, rows=None, _lib_override=None,
            window=0):
    """Parallax forward by the plain definition.

    q, r : [B, Hq, Tq, d]; k, v : [B, Hkv, Lk, d]; all float64 or all float32 numpy arrays
    (float32 holds bf16/fp32 inputs exactly; it is widened to double before any arithmetic).
    causal : key j allowed iff j <= i + (Lk - Tq) (queries are the last Tq positions; needs
             Tq <= Lk; the square case is j <= i); else j < seq_lens[b] (default Lk).
    window : 0 = none; W > 0: a row sees only the last W of its allowed keys (the query's own
             position and the W - 1 before it); causal or Tq == 1 only.
    rows : optional int array [n, 3] of (b, h, i); then the result is [n, d].
    Returns float64.
    """
    lib = _lib_override if _lib_override is not None else _load()
    dt = np.float64 if q.dtype == np.float64 else np.float32
    q, r, k, v = (np.ascontiguousarray(x, dtype=dt) for x in (q, r, k, v))
    B, Hq, Tq, d = q.shape
    Bk, Hkv, Lk, dk = k.shape
    assert r.shape == q.shape and v.shape == k.shape and Bk == B and dk == d
    sl = None
    if seq_lens is not None:
        sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
        assert sl.shape == (B,)
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        assert rows.ndim == 2 and rows.shape[1] == 3
        out = np.zeros((rows.shape[0], d), dtype=np.float64)
        n_rows = rows.shape[0]
    else:
        out = np.zeros((B, Hq, Tq, d), dtype=np.float64)
        n_rows = 0
    fn = lib.plx_oracle_f64 if dt == np.float64 else lib.plx_oracle_f32in
    rc = fn(q.ctypes.data, r.ctypes.data, k.ctypes.data, v.ctypes.data, out.ctypes.data,
            B, Hq, Hkv, Tq, Lk, d, float(scale), int(bool(causal)),
            sl.ctypes.data if sl is not None else None,
            rows.ctypes.data if rows is not None else None, n_rows, int(window))
    if rc != 0:
        raise ValueError("parallax oracle rejected its arguments (rc=%d)" % rc)
    return out
