"""ctypes binding of the C oracle (oracle/varlen_attn_oracle.c).  TEST INFRASTRUCTURE ONLY.

Argument marshalling only; the arithmetic is in the C file.  Inputs are numpy float32
arrays holding bf16-representable values (any float32 works), outputs are float64.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "varlen_attn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_attn.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (-O2, no fast-math, OpenMP)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        i32p = ctypes.POINTER(ctypes.c_int32)
        i64p = ctypes.POINTER(ctypes.c_int64)
        ci, cd = ctypes.c_int, ctypes.c_double
        lib.oracle_varlen_attn_fwd.argtypes = [f32p, f32p, f32p, i32p, ci, ci, ci, ci, ci, cd, f64p, f64p]
        lib.oracle_varlen_attn_fwd.restype = ci
        lib.oracle_varlen_attn_fwd_rows.argtypes = [f32p, f32p, f32p, i32p, ci, ci, ci, ci, ci, cd,
                                                    i64p, ctypes.c_int64, f64p, f64p]
        lib.oracle_varlen_attn_fwd_rows.restype = ci
        lib.oracle_varlen_attn_bwd.argtypes = [f32p, f32p, f32p, f32p, i32p, ci, ci, ci, ci, ci, cd,
                                               f64p, f64p, f64p]
        lib.oracle_varlen_attn_bwd.restype = ci
        lib.oracle_varlen_attn_bwd_saved_o.argtypes = [f32p, f32p, f32p, f32p, f64p, i32p, ci, ci, ci, ci, ci, cd,
                                                       f64p, f64p, f64p]
        lib.oracle_varlen_attn_bwd_saved_o.restype = ci
        lib.oracle_varlen_attn_bwd_q_rows.argtypes = [f32p, f32p, f32p, f32p, f64p, i32p, ci, ci, ci, ci, ci, cd,
                                                      i64p, ctypes.c_int64, f64p]
        lib.oracle_varlen_attn_bwd_q_rows.restype = ci
        lib.oracle_varlen_attn_bwd_kv_rows.argtypes = [f32p, f32p, f32p, f32p, f64p, i32p, ci, ci, ci, ci, ci, cd,
                                                       ci, i64p, ctypes.c_int64, f64p, f64p]
        lib.oracle_varlen_attn_bwd_kv_rows.restype = ci
        lib.oracle_num_threads.restype = ci
        lib.oracle_attn_merge.argtypes = [f32p, f64p, ci, ci, ci, ci, f64p, f64p]
        lib.oracle_attn_merge.restype = ci
        _lib = lib
    return _lib


def _f32(a, shape):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if a.shape != shape:
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


def _ptr(a, ty):
    return a.ctypes.data_as(ctypes.POINTER(ty))


def _shapes(q, k, cu):
    cu = np.ascontiguousarray(cu, dtype=np.int32)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    if cu.ndim != 1 or cu.size < 1 or int(cu[-1]) != T:
        raise ValueError("cu_seqlens must be 1-D with cu[-1] == total tokens")
    return cu, T, Hq, Hkv, D


def num_threads():
    return int(_load().oracle_num_threads())


def fwd(q, k, v, cu_seqlens, causal, scale):
    """O [T,Hq,D] float64 and LSE [Hq,T] float64 (natural log) for every packed row."""
    lib = _load()
    cu, T, Hq, Hkv, D = _shapes(q, k, cu_seqlens)
    q, k, v = _f32(q, (T, Hq, D)), _f32(k, (T, Hkv, D)), _f32(v, (T, Hkv, D))
    o = np.empty((T, Hq, D), np.float64)
    lse = np.empty((Hq, T), np.float64)
    rc = lib.oracle_varlen_attn_fwd(_ptr(q, ctypes.c_float), _ptr(k, ctypes.c_float),
                                    _ptr(v, ctypes.c_float), _ptr(cu, ctypes.c_int32), cu.size - 1,
                                    Hq, Hkv, D, int(bool(causal)), float(scale),
                                    _ptr(o, ctypes.c_double), _ptr(lse, ctypes.c_double))
    if rc:
        raise RuntimeError(f"oracle fwd failed with status {rc}")
    return o, lse


def fwd_rows(q, k, v, cu_seqlens, causal, scale, rows):
    """O [n,Hq,D] and LSE [n,Hq] float64 for the listed packed rows only (exact per row)."""
    lib = _load()
    cu, T, Hq, Hkv, D = _shapes(q, k, cu_seqlens)
    q, k, v = _f32(q, (T, Hq, D)), _f32(k, (T, Hkv, D)), _f32(v, (T, Hkv, D))
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    o = np.empty((rows.size, Hq, D), np.float64)
    lse = np.empty((rows.size, Hq), np.float64)
    rc = lib.oracle_varlen_attn_fwd_rows(_ptr(q, ctypes.c_float), _ptr(k, ctypes.c_float),
                                         _ptr(v, ctypes.c_float), _ptr(cu, ctypes.c_int32),
                                         cu.size - 1, Hq, Hkv, D, int(bool(causal)), float(scale),
                                         _ptr(rows, ctypes.c_int64), rows.size,
                                         _ptr(o, ctypes.c_double), _ptr(lse, ctypes.c_double))
    if rc:
        raise RuntimeError(f"oracle fwd_rows failed with status {rc}")
    return o, lse


def _saved_o(o_saved, shape):
    """The stored forward output as float64 [T,Hq,D] (a bf16 or fp32 value converts exactly), or None."""
    if o_saved is None:
        return None
    o_saved = np.ascontiguousarray(o_saved, dtype=np.float64)
    if o_saved.shape != shape:
        raise ValueError(f"expected o_saved of shape {shape}, got {o_saved.shape}")
    return o_saved


def bwd(q, k, v, dout, cu_seqlens, causal, scale, o_saved=None):
    """dQ [T,Hq,D], dK, dV [T,Hkv,D] float64, from the oracle's own fp64 forward.  With o_saved (the
    forward output as a caller stored it, [T,Hq,D]) Delta = <dO, O> is formed from that instead of the
    oracle's own O; everything else stays the definition."""
    lib = _load()
    cu, T, Hq, Hkv, D = _shapes(q, k, cu_seqlens)
    q, k, v = _f32(q, (T, Hq, D)), _f32(k, (T, Hkv, D)), _f32(v, (T, Hkv, D))
    dout = _f32(dout, (T, Hq, D))
    o_saved = _saved_o(o_saved, (T, Hq, D))
    dq = np.empty((T, Hq, D), np.float64)
    dk = np.empty((T, Hkv, D), np.float64)
    dv = np.empty((T, Hkv, D), np.float64)
    head = (_ptr(q, ctypes.c_float), _ptr(k, ctypes.c_float), _ptr(v, ctypes.c_float), _ptr(dout, ctypes.c_float))
    tail = (_ptr(cu, ctypes.c_int32), cu.size - 1, Hq, Hkv, D, int(bool(causal)), float(scale),
            _ptr(dq, ctypes.c_double), _ptr(dk, ctypes.c_double), _ptr(dv, ctypes.c_double))
    if o_saved is None:
        rc = lib.oracle_varlen_attn_bwd(*head, *tail)
    else:
        rc = lib.oracle_varlen_attn_bwd_saved_o(*head, _ptr(o_saved, ctypes.c_double), *tail)
    if rc:
        raise RuntimeError(f"oracle bwd failed with status {rc}")
    return dq, dk, dv


def bwd_q_rows(q, k, v, dout, cu_seqlens, causal, scale, rows, o_saved=None):
    """dQ [n,Hq,D] float64 for the listed packed query rows only (exact per row at any sample length)."""
    lib = _load()
    cu, T, Hq, Hkv, D = _shapes(q, k, cu_seqlens)
    q, k, v = _f32(q, (T, Hq, D)), _f32(k, (T, Hkv, D)), _f32(v, (T, Hkv, D))
    dout = _f32(dout, (T, Hq, D))
    o_saved = _saved_o(o_saved, (T, Hq, D))
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    dq = np.empty((rows.size, Hq, D), np.float64)
    rc = lib.oracle_varlen_attn_bwd_q_rows(
        _ptr(q, ctypes.c_float), _ptr(k, ctypes.c_float), _ptr(v, ctypes.c_float), _ptr(dout, ctypes.c_float),
        None if o_saved is None else _ptr(o_saved, ctypes.c_double), _ptr(cu, ctypes.c_int32), cu.size - 1,
        Hq, Hkv, D, int(bool(causal)), float(scale), _ptr(rows, ctypes.c_int64), rows.size,
        _ptr(dq, ctypes.c_double))
    if rc:
        raise RuntimeError(f"oracle bwd_q_rows failed with status {rc}")
    return dq


def bwd_kv_rows(q, k, v, dout, cu_seqlens, causal, scale, kv_head, rows, o_saved=None):
    """dK, dV [n,D] float64 of kv head `kv_head` for the listed packed key rows only (exact per row; the
    statistics of every query row of the rows' samples are evaluated on the way)."""
    lib = _load()
    cu, T, Hq, Hkv, D = _shapes(q, k, cu_seqlens)
    q, k, v = _f32(q, (T, Hq, D)), _f32(k, (T, Hkv, D)), _f32(v, (T, Hkv, D))
    dout = _f32(dout, (T, Hq, D))
    o_saved = _saved_o(o_saved, (T, Hq, D))
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    dk = np.empty((rows.size, D), np.float64)
    dv = np.empty((rows.size, D), np.float64)
    rc = lib.oracle_varlen_attn_bwd_kv_rows(
        _ptr(q, ctypes.c_float), _ptr(k, ctypes.c_float), _ptr(v, ctypes.c_float), _ptr(dout, ctypes.c_float),
        None if o_saved is None else _ptr(o_saved, ctypes.c_double), _ptr(cu, ctypes.c_int32), cu.size - 1,
        Hq, Hkv, D, int(bool(causal)), float(scale), int(kv_head), _ptr(rows, ctypes.c_int64), rows.size,
        _ptr(dk, ctypes.c_double), _ptr(dv, ctypes.c_double))
    if rc:
        raise RuntimeError(f"oracle bwd_kv_rows failed with status {rc}")
    return dk, dv


def merge(o_parts, lse_parts):
    """Combine partial results over disjoint key shards: o_parts [P,T,H,D], lse_parts [P,H,T] (-inf = the
    shard held no key for that row).  Returns (O float64 [T,H,D], LSE float64 [H,T])."""
    o_parts = np.ascontiguousarray(o_parts, dtype=np.float32)
    P, T, H, D = o_parts.shape
    lse_parts = np.ascontiguousarray(lse_parts, dtype=np.float64)
    if lse_parts.shape != (P, H, T):
        raise ValueError(f"expected lse_parts of shape {(P, H, T)}, got {lse_parts.shape}")
    o = np.empty((T, H, D), dtype=np.float64)
    lse = np.empty((H, T), dtype=np.float64)
    rc = _load().oracle_attn_merge(_ptr(o_parts, ctypes.c_float), _ptr(lse_parts, ctypes.c_double), P, T, H, D,
                                   _ptr(o, ctypes.c_double), _ptr(lse, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"oracle_attn_merge failed with code {rc}")
    return o, lse
