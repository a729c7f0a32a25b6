"""fp64 CPU oracle for the TokenSwift decode-attention hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes front end of ``ts_oracle.c`` (which carries the citations of the passages each
function follows).  Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package; the GPU library never does, and this package never imports the GPU
library.  Arrays of bf16 values are passed as ``numpy.uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ts_oracle.c")
_LIB = os.path.join(_HERE, "libts_oracle.so")


def build(force: bool = False) -> str:
    """Compile ts_oracle.c with gcc (OpenMP) into libts_oracle.so beside it."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
               _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f64p = ctypes.POINTER(ctypes.c_double)
        i64 = ctypes.c_int64
        ci = ctypes.c_int
        lib.oracle_num_threads.restype = ci
        lib.oracle_set_threads.argtypes = [ci]
        lib.oracle_set_threads.restype = None
        lib.oracle_chunk_scores.argtypes = [u16p, u16p, ci, ci, i64, ci, i64, i64, ci,
                                            ctypes.c_double, f64p]
        lib.oracle_topk_chunks.argtypes = [f64p, ci, i64, ci, ci, i32p]
        lib.oracle_partial_attn.argtypes = [u16p, u16p, u16p, ci, ci, i64, ci, i64, i64, i32p, ci,
                                            ci, ctypes.c_double, f64p, f64p]
        lib.oracle_tree_verify.argtypes = [u16p, u16p, u16p, u16p, u16p, i32p, ci, ci, ci, i64, ci,
                                           i64, i64, ctypes.c_double, i32p, i32p, i64, f64p, f64p]
        lib.oracle_combine.argtypes = [f64p, f64p, f64p, ci, ci, f64p, f64p]
        for name in ("oracle_chunk_scores", "oracle_topk_chunks", "oracle_partial_attn",
                     "oracle_tree_verify", "oracle_combine"):
            getattr(lib, name).restype = ci
        _lib = lib
    return _lib


def _u16(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("bf16 arrays are passed as uint16 bit patterns, got %s" % a.dtype)
    return a


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype)) if a is not None else None


def _check(rc, what):
    if rc != 0:
        raise ValueError("%s: invalid arguments (code %d)" % (what, rc))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_threads(n: int) -> None:
    _load().oracle_set_threads(int(n))


def _kv_strides(k):
    """k is [n_kv_heads, n_tokens, d] contiguous in d; returns element strides."""
    if k.ndim != 3:
        raise ValueError("cache must be [n_kv_heads, n_tokens, d]")
    es = k.itemsize
    if k.strides[2] != es:
        raise ValueError("last axis must be contiguous")
    return k.strides[0] // es, k.strides[1] // es


def chunk_scores(q, k, chunk, scale):
    """q [Hq,d] u16, k [Hkv,N,d] u16 -> scores [Hkv, ceil(N/chunk)] float64."""
    q = _u16(q)
    if k.dtype != np.uint16:
        raise TypeError("k must be uint16")
    hq, d = q.shape
    hkv, n, d2 = k.shape
    assert d == d2
    sh, st = _kv_strides(k)
    n_chunks = (n + chunk - 1) // chunk
    out = np.empty((hkv, n_chunks), dtype=np.float64)
    rc = _load().oracle_chunk_scores(_ptr(q, ctypes.c_uint16), _ptr(k, ctypes.c_uint16), hq, hkv,
                                     n, d, sh, st, int(chunk), float(scale),
                                     _ptr(out, ctypes.c_double))
    _check(rc, "oracle_chunk_scores")
    return out


def topk_chunks(scores, n_sink, k):
    """scores [Hkv, n_chunks] (any float dtype, widened exactly) -> idx [Hkv, n_sink+k] int32."""
    s = np.ascontiguousarray(np.asarray(scores).astype(np.float64))
    hkv, n_chunks = s.shape
    idx = np.empty((hkv, n_sink + k), dtype=np.int32)
    rc = _load().oracle_topk_chunks(_ptr(s, ctypes.c_double), hkv, n_chunks, int(n_sink), int(k),
                                    _ptr(idx, ctypes.c_int32))
    _check(rc, "oracle_topk_chunks")
    return idx


def partial_attn(q, k, v, chunk_idx, chunk, scale):
    """q [Hq,d], k/v [Hkv,N,d] u16, chunk_idx [Hkv,n_sel] int32 -> (out [Hq,d], lse [Hq]) float64."""
    q = _u16(q)
    hq, d = q.shape
    hkv, n, _ = k.shape
    sh, st = _kv_strides(k)
    assert _kv_strides(v) == (sh, st), "k and v must share strides"
    idx = np.ascontiguousarray(chunk_idx, dtype=np.int32)
    assert idx.shape[0] == hkv
    out = np.empty((hq, d), dtype=np.float64)
    lse = np.empty((hq,), dtype=np.float64)
    rc = _load().oracle_partial_attn(_ptr(q, ctypes.c_uint16), _ptr(k, ctypes.c_uint16),
                                     _ptr(v, ctypes.c_uint16), hq, hkv, n, d, sh, st,
                                     _ptr(idx, ctypes.c_int32), idx.shape[1], int(chunk),
                                     float(scale), _ptr(out, ctypes.c_double),
                                     _ptr(lse, ctypes.c_double))
    _check(rc, "oracle_partial_attn")
    return out, lse


def tree_verify(q_tree, k, v, k_tree, v_tree, parent, scale, rows=None):
    """q_tree [T,Hq,d], k/v [Hkv,N,d] (N may be 0), k_tree/v_tree [T,Hkv,d] u16, parent [T].

    rows=None -> (out [T,Hq,d], lse [T,Hq]); rows=[(node, head), ...] -> (out [n,d], lse [n]).
    """
    q_tree = _u16(q_tree)
    k_tree = _u16(k_tree)
    v_tree = _u16(v_tree)
    t, hq, d = q_tree.shape
    hkv = k_tree.shape[1]
    n = 0 if k is None else k.shape[1]
    if n > 0:
        sh, st = _kv_strides(k)
        assert _kv_strides(v) == (sh, st)
        kp, vp = _ptr(k, ctypes.c_uint16), _ptr(v, ctypes.c_uint16)
    else:
        sh = st = 0
        kp = vp = None
    par = np.ascontiguousarray(parent, dtype=np.int32)
    assert par.shape == (t,)
    if rows is None:
        out = np.empty((t, hq, d), dtype=np.float64)
        lse = np.empty((t, hq), dtype=np.float64)
        rn = rh = None
        n_rows = -1
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 2)
        rn = np.ascontiguousarray(rows[:, 0])
        rh = np.ascontiguousarray(rows[:, 1])
        n_rows = rows.shape[0]
        out = np.empty((n_rows, d), dtype=np.float64)
        lse = np.empty((n_rows,), dtype=np.float64)
    rc = _load().oracle_tree_verify(_ptr(q_tree, ctypes.c_uint16), kp, vp,
                                    _ptr(k_tree, ctypes.c_uint16), _ptr(v_tree, ctypes.c_uint16),
                                    _ptr(par, ctypes.c_int32), t, hq, hkv, n, d, sh, st,
                                    float(scale), _ptr(rn, ctypes.c_int32) if rn is not None else None,
                                    _ptr(rh, ctypes.c_int32) if rh is not None else None, n_rows,
                                    _ptr(out, ctypes.c_double), _ptr(lse, ctypes.c_double))
    _check(rc, "oracle_tree_verify")
    return out, lse


def combine(m, l, o):
    """m [P], l [P], o [P,d] float64 -> (out [d], lse)."""
    m = np.ascontiguousarray(m, dtype=np.float64)
    l = np.ascontiguousarray(l, dtype=np.float64)
    o = np.ascontiguousarray(o, dtype=np.float64)
    p, d = o.shape
    out = np.empty((d,), dtype=np.float64)
    lse = np.empty((1,), dtype=np.float64)
    rc = _load().oracle_combine(_ptr(m, ctypes.c_double), _ptr(l, ctypes.c_double),
                                _ptr(o, ctypes.c_double), p, d, _ptr(out, ctypes.c_double),
                                _ptr(lse, ctypes.c_double))
    _check(rc, "oracle_combine")
    return out, float(lse[0])
