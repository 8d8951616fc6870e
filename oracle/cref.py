"""ctypes front end of the plain-C fp64 oracle (oracle/ref_attention.c).

Test infrastructure only.  Same definition as oracle/ref_attention.py, usable at
the large configurations because it is compiled and threaded.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.ref_prefix_shared_attention.restype = ctypes.c_int
        lib.ref_prefix_shared_attention.argtypes = [
            fp, fp, fp, fp, fp, ctypes.POINTER(ctypes.c_int32), ctypes.c_int, ctypes.c_int64,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
            ctypes.POINTER(ctypes.c_int64), ctypes.c_int64, dp, dp, ctypes.c_int]
        lib.ref_prefix_shared_attention_backward.restype = ctypes.c_int
        lib.ref_prefix_shared_attention_backward.argtypes = [
            fp, fp, fp, fp, fp, fp, ctypes.POINTER(ctypes.c_int32), ctypes.c_int, ctypes.c_int64,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
            ctypes.POINTER(ctypes.c_int64), ctypes.c_int64, dp, dp, dp, dp, dp, ctypes.c_int]
        _lib = lib
    return _lib


def _f32(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    return x, x.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def prefix_shared_attention(q, k_prefix, v_prefix, k_suffix, v_suffix, suffix_lens, scale,
                            rows=None, num_threads=0):
    """Returns (out, lse, threads_used).

    rows=None: out [T,Hq,D], lse [Hq,T] for every packed row.
    rows=array: out [n,Hq,D], lse [Hq,n] for those packed token rows only.
    Inputs are float32 arrays holding the exact values both sides consume.
    """
    lib = _load()
    q, qp = _f32(q)
    T, Hq, D = q.shape
    k_prefix, kpp = _f32(k_prefix)
    v_prefix, vpp = _f32(v_prefix)
    k_suffix, ksp = _f32(k_suffix)
    v_suffix, vsp = _f32(v_suffix)
    P, Hkv = int(k_prefix.shape[0]), int(k_suffix.shape[1])
    lens = np.ascontiguousarray(suffix_lens, dtype=np.int32)
    assert int(lens.sum()) == T
    if rows is None:
        n, rp = T, None
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        n, rp = len(rows), rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
    out = np.empty((n, Hq, D), dtype=np.float64)
    lse = np.empty((Hq, n), dtype=np.float64)
    rc = lib.ref_prefix_shared_attention(
        qp, kpp, vpp, ksp, vsp, lens.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), len(lens), P,
        Hq, Hkv, D, float(scale), rp, n, out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
        lse.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), int(num_threads))
    if rc < 0:
        raise RuntimeError(f"ref_prefix_shared_attention failed with {rc}")
    return out, lse, rc


def prefix_shared_attention_backward(q, k_prefix, v_prefix, k_suffix, v_suffix, suffix_lens, scale, d_out,
                                     rows=None, num_threads=0):
    """Gradients of L = sum(d_out * out).

    rows=None: returns (dq [T,Hq,D], dk_prefix, dv_prefix [P,Hkv,D], dk_suffix, dv_suffix [T,Hkv,D], threads).
    rows=array: returns (dq [n,Hq,D] for those packed token rows, threads); key/value gradients are not computed.
    """
    lib = _load()
    q, qp = _f32(q)
    T, Hq, D = q.shape
    k_prefix, kpp = _f32(k_prefix)
    v_prefix, vpp = _f32(v_prefix)
    k_suffix, ksp = _f32(k_suffix)
    v_suffix, vsp = _f32(v_suffix)
    d_out, dop = _f32(d_out)
    assert d_out.shape == q.shape
    P, Hkv = int(k_prefix.shape[0]), int(k_suffix.shape[1])
    lens = np.ascontiguousarray(suffix_lens, dtype=np.int32)
    assert int(lens.sum()) == T
    dptr = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))
    if rows is None:
        n, rp = T, None
        grads = [np.empty((P, Hkv, D)), np.empty((P, Hkv, D)), np.empty((T, Hkv, D)), np.empty((T, Hkv, D))]
        gp = [dptr(a) for a in grads]
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        n, rp = len(rows), rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
        grads, gp = [], [None] * 4
    dq = np.empty((n, Hq, D), dtype=np.float64)
    rc = lib.ref_prefix_shared_attention_backward(
        qp, kpp, vpp, ksp, vsp, dop, lens.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), len(lens), P,
        Hq, Hkv, D, float(scale), rp, n, dptr(dq), *gp, int(num_threads))
    if rc < 0:
        raise RuntimeError(f"ref_prefix_shared_attention_backward failed with {rc}")
    return (dq, *grads, rc)
