"""ORACLE -- test infrastructure only: ctypes wrapper over oracle/attention.c (fp64, CPU).

seq_attn_fwd / seq_attn_bwd     the definition: causal softmax attention of one whole sequence
chunk_attn_fwd / chunk_attn_bwd the chunked method: segments with optional retained prefix keys
See attention.c's header for the formulas and the paper passages they follow.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle_attention.so")
_SRC = os.path.join(_HERE, "attention.c")


def build(force=False):
    """Compile attention.c with gcc (OpenMP).  No -march flag: the library travels between hosts."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               _SRC, "-o", _SO, "-lm"])
    return _SO


_lib = None


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        lib = ctypes.CDLL(_SO)
        i64, f64, p = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.orc_num_threads.restype = ctypes.c_int
        lib.orc_seq_attn_fwd.argtypes = [i64, i64, i64, i64, f64, p, p, p, p, p]
        lib.orc_seq_attn_fwd.restype = None
        lib.orc_seq_attn_bwd.argtypes = [i64, i64, i64, i64, f64] + [p] * 9
        lib.orc_seq_attn_bwd.restype = None
        lib.orc_chunk_attn_fwd.argtypes = [i64, p, p, i64, i64, i64, f64, p, p, p, p, p]
        lib.orc_chunk_attn_fwd.restype = ctypes.c_int
        lib.orc_chunk_attn_bwd.argtypes = [i64, p, p, i64, i64, i64, f64] + [p] * 9
        lib.orc_chunk_attn_bwd.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads():
    return int(_load().orc_num_threads())


def _c(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def seq_attn_fwd(q, k, v, scale):
    """q [L,Hq,D], k,v [L,Hkv,D] -> o [L,Hq,D], lse [Hq,L]."""
    q, k, v = _c(q), _c(k), _c(v)
    L, Hq, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (L, Hkv, D) and v.shape == (L, Hkv, D) and Hq % Hkv == 0
    o = np.empty_like(q)
    lse = np.empty((Hq, L), dtype=np.float64)
    _load().orc_seq_attn_fwd(L, Hq, Hkv, D, float(scale), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse))
    return o, lse


def seq_attn_bwd(q, k, v, o, lse, d_o, scale):
    """-> dq [L,Hq,D], dk, dv [L,Hkv,D]."""
    q, k, v, o, lse, d_o = _c(q), _c(k), _c(v), _c(o), _c(lse), _c(d_o)
    L, Hq, D = q.shape
    Hkv = k.shape[1]
    dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
    _load().orc_seq_attn_bwd(L, Hq, Hkv, D, float(scale), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse),
                             _ptr(d_o), _ptr(dq), _ptr(dk), _ptr(dv))
    return dq, dk, dv


def _cu(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def chunk_attn_fwd(q, k, v, cu_q, cu_k, scale):
    """q [Tq,Hq,D], k,v [Tk,Hkv,D]; cu_q, cu_k [n_seg+1] -> o [Tq,Hq,D], lse [Hq,Tq]."""
    q, k, v, cu_q, cu_k = _c(q), _c(k), _c(v), _cu(cu_q), _cu(cu_k)
    Tq, Hq, D = q.shape
    Tk, Hkv, _ = k.shape
    n_seg = len(cu_q) - 1
    assert len(cu_k) == n_seg + 1 and cu_q[0] == 0 and cu_k[0] == 0
    assert cu_q[-1] == Tq and cu_k[-1] == Tk and v.shape == k.shape and Hq % Hkv == 0
    o = np.empty_like(q)
    lse = np.empty((Hq, Tq), dtype=np.float64)
    rc = _load().orc_chunk_attn_fwd(n_seg, _ptr(cu_q), _ptr(cu_k), Hq, Hkv, D, float(scale),
                                    _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse))
    if rc != 0:
        raise ValueError("a segment has more query rows than key rows")
    return o, lse


def chunk_attn_bwd(q, k, v, o, lse, d_o, cu_q, cu_k, scale, dk, dv):
    """Adds this chunk's contributions into dk, dv (fp64 [Tk,Hkv,D], modified in place); returns dq."""
    q, k, v, o, lse, d_o, cu_q, cu_k = _c(q), _c(k), _c(v), _c(o), _c(lse), _c(d_o), _cu(cu_q), _cu(cu_k)
    Tq, Hq, D = q.shape
    Tk, Hkv, _ = k.shape
    n_seg = len(cu_q) - 1
    assert cu_q[-1] == Tq and cu_k[-1] == Tk
    for g in (dk, dv):
        assert g.dtype == np.float64 and g.flags.c_contiguous and g.shape == (Tk, Hkv, D)
    dq = np.empty_like(q)
    rc = _load().orc_chunk_attn_bwd(n_seg, _ptr(cu_q), _ptr(cu_k), Hq, Hkv, D, float(scale),
                                    _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o),
                                    _ptr(dq), _ptr(dk), _ptr(dv))
    if rc != 0:
        raise ValueError("a segment has more query rows than key rows")
    return dq
