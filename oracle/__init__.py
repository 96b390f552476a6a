"""fp64 CPU reference for attention forward -- TEST INFRASTRUCTURE, not the product.

Thin ctypes binding of ``attn_ref.c`` (the plain definition of Section 2 of the
paper: S = Q K^T, P = softmax(S), O = P V, plus scale, GQA, causal mask and LSE as
the library boundary states them).  Only ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py`` may import this package; the product
package never does.  Nothing here touches a GPU or the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_ref.c")
_LIB = os.path.join(_HERE, "liboracle_attn.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile attn_ref.c with gcc (plain -O2, no fast-math) and return the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i, d, p = ctypes.c_int, ctypes.c_double, ctypes.c_void_p
        lib.attn_ref_f64.restype = i
        lib.attn_ref_f64.argtypes = [p, p, p, p, p, i, i, i, i, i, i, i, d, p, i]
        lib.attn_ref_f64_from_f64.restype = i
        lib.attn_ref_f64_from_f64.argtypes = [p, p, p, p, p, i, i, i, i, i, i, i, d, p, i]
        lib.attn_ref_row_probs_f64.restype = i
        lib.attn_ref_row_probs_f64.argtypes = [p, p, p, i, i, i, i, i, i, i, d, i, i, i, p, p, p]
        _lib = lib
    return _lib


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _dims(q, k, v):
    B, Hq, Sq, D = q.shape
    Bk, Hkv, Sk, Dk = k.shape
    if v.shape != k.shape or Bk != B or Dk != D:
        raise ValueError("inconsistent q/k/v shapes")
    return B, Hq, Hkv, Sq, Sk, D


def _rows_arg(rows, B, Hq):
    if rows is None:
        return None, 0
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    if rows.ndim == 1:  # same rows for every (b, h)
        rows = np.ascontiguousarray(np.broadcast_to(rows, (B * Hq, rows.shape[0])))
    rows = rows.reshape(B * Hq, -1)
    return rows, rows.shape[1]


def attn_ref(q, k, v, causal: bool, scale: float, rows=None):
    """Reference O (fp64) and LSE (fp64).

    q [B,Hq,Sq,D], k/v [B,Hkv,Sk,D]: either uint16 arrays of bf16 bit patterns or
    float64 arrays.  rows: None (all query rows), a 1-D list used for every (b,h),
    or an int array [B*Hq, n] / [B,Hq,n] of query indices per head.
    Returns (o [B,Hq,R,D], lse [B,Hq,R]) with R = Sq or n.
    """
    lib = _load()
    B, Hq, Hkv, Sq, Sk, D = _dims(q, k, v)
    rows_a, nrows = _rows_arg(rows, B, Hq)
    R = nrows if rows_a is not None else Sq
    o = np.empty((B, Hq, R, D), dtype=np.float64)
    lse = np.empty((B, Hq, R), dtype=np.float64)
    if q.dtype == np.uint16:
        fn, dt = lib.attn_ref_f64, np.uint16
    elif q.dtype == np.float64:
        fn, dt = lib.attn_ref_f64_from_f64, np.float64
    else:
        raise TypeError("q/k/v must be uint16 (bf16 bits) or float64")
    q, k, v = (np.ascontiguousarray(x, dtype=dt) for x in (q, k, v))
    rc = fn(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), B, Hq, Hkv, Sq, Sk, D,
            int(bool(causal)), float(scale), _ptr(rows_a) if rows_a is not None else None, nrows)
    if rc != 0:
        raise RuntimeError("attn_ref failed with code %d" % rc)
    return o, lse


def attn_ref_row_probs(q, k, v, causal: bool, scale: float, b: int, h: int, i: int):
    """Softmax probabilities [Sk], O row [D] and LSE of one query row (bf16-bit inputs)."""
    lib = _load()
    B, Hq, Hkv, Sq, Sk, D = _dims(q, k, v)
    q, k, v = (np.ascontiguousarray(x, dtype=np.uint16) for x in (q, k, v))
    probs = np.empty(Sk, dtype=np.float64)
    orow = np.empty(D, dtype=np.float64)
    lse = np.empty(1, dtype=np.float64)
    rc = lib.attn_ref_row_probs_f64(_ptr(q), _ptr(k), _ptr(v), B, Hq, Hkv, Sq, Sk, D,
                                    int(bool(causal)), float(scale), b, h, i,
                                    _ptr(probs), _ptr(orow), _ptr(lse))
    if rc != 0:
        raise RuntimeError("attn_ref_row_probs failed with code %d" % rc)
    return probs, orow, float(lse[0])
