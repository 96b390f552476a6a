"""fp64 CPU references -- TEST INFRASTRUCTURE, not the product.

Thin ctypes bindings of ``attn_ref.c`` (the plain definition in the "Motivating Example" section of the
paper: S = Q K^T, P = softmax(S), O = P V, plus scale, GQA, causal mask and LSE as
the library boundary states them) and of ``gemm_ref.c`` (the bf16 matrix product of
the paper's GEMM workload, Evaluation / "Kernel Performance", as three nested loops) and of ``moe_ref.c`` (the
block-quantized FP8 mixture-of-experts feed-forward of the same subsection, step by step).  Only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import this
package; the product package never does.  Nothing here touches a GPU or the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_ref.c")
_LIB = os.path.join(_HERE, "liboracle_attn.so")
_GEMM_SRC = os.path.join(_HERE, "gemm_ref.c")
_GEMM_LIB = os.path.join(_HERE, "liboracle_gemm.so")
_MOE_SRC = os.path.join(_HERE, "moe_ref.c")
_MOE_LIB = os.path.join(_HERE, "liboracle_moe.so")
_lib = None
_gemm_lib = None
_moe_lib = None


def _compile(src: str, lib: str, force: bool) -> str:
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(src):
        tmp = lib + ".tmp.%d" % os.getpid()
        # -ffp-contract=off: the fp32 steps of the quantization recipes must not be fused
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", tmp, src, "-lm"])
        os.replace(tmp, lib)
    return lib


def build(force: bool = False) -> str:
    """Compile the C references with gcc (plain -O2, no fast-math); returns the attention .so path."""
    _compile(_GEMM_SRC, _GEMM_LIB, force)
    _compile(_MOE_SRC, _MOE_LIB, force)
    return _compile(_SRC, _LIB, force)


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


def _load_gemm():
    global _gemm_lib
    if _gemm_lib is None:
        lib = ctypes.CDLL(_compile(_GEMM_SRC, _GEMM_LIB, False))
        i, ll, p = ctypes.c_int, ctypes.c_longlong, ctypes.c_void_p
        lib.gemm_ref_f64.restype = i
        lib.gemm_ref_f64.argtypes = [p, p, p, p, i, i, i, ll, ll, i]
        lib.gemm_ref_f64_samples.restype = i
        lib.gemm_ref_f64_samples.argtypes = [p, p, p, p, i, p, p, i, i, i, ll, ll, i]
        _gemm_lib = lib
    return _gemm_lib


def _gemm_dims(a, b, b_is_nk):
    if a.dtype != np.uint16 or b.dtype != np.uint16 or a.ndim != 2 or b.ndim != 2:
        raise TypeError("a, b must be 2-D uint16 arrays of bf16 bit patterns")
    if a.strides[1] != 2 or b.strides[1] != 2 or a.strides[0] % 2 or b.strides[0] % 2:
        raise ValueError("rows of a and b must be contiguous")
    M, K = a.shape
    N = b.shape[0] if b_is_nk else b.shape[1]
    if (b.shape[1] if b_is_nk else b.shape[0]) != K:
        raise ValueError("inner dimensions differ")
    return M, N, K, a.strides[0] // 2, b.strides[0] // 2


def gemm_ref(a, b, b_is_nk: bool = False):
    """C = A B in fp64 and the absolute sums sum_k |a_ik||b_kj| (both [M,N]).

    a [M,K], b [K,N] (or [N,K] if b_is_nk): uint16 arrays of bf16 bits; rows contiguous, row
    pitch free (slices of wider arrays are fine).
    """
    lib = _load_gemm()
    M, N, K, lda, ldb = _gemm_dims(a, b, b_is_nk)
    c = np.empty((M, N), dtype=np.float64)
    cabs = np.empty((M, N), dtype=np.float64)
    rc = lib.gemm_ref_f64(_ptr(a), _ptr(b), _ptr(c), _ptr(cabs), M, N, K, lda, ldb, int(bool(b_is_nk)))
    if rc != 0:
        raise RuntimeError("gemm_ref failed with code %d" % rc)
    return c, cabs


def gemm_ref_samples(a, b, si, sj, b_is_nk: bool = False):
    """c[si[t], sj[t]] and its absolute sum for each sampled output t."""
    lib = _load_gemm()
    M, N, K, lda, ldb = _gemm_dims(a, b, b_is_nk)
    si = np.ascontiguousarray(si, dtype=np.int32)
    sj = np.ascontiguousarray(sj, dtype=np.int32)
    if si.shape != sj.shape or si.ndim != 1:
        raise ValueError("si, sj must be 1-D and of equal length")
    out = np.empty(si.shape[0], dtype=np.float64)
    outabs = np.empty(si.shape[0], dtype=np.float64)
    rc = lib.gemm_ref_f64_samples(_ptr(a), _ptr(b), _ptr(si), _ptr(sj), si.shape[0], _ptr(out), _ptr(outabs),
                                  M, N, K, lda, ldb, int(bool(b_is_nk)))
    if rc != 0:
        raise RuntimeError("gemm_ref_samples failed with code %d" % rc)
    return out, outabs


def _load_moe():
    global _moe_lib
    if _moe_lib is None:
        lib = ctypes.CDLL(_compile(_MOE_SRC, _MOE_LIB, False))
        i, p = ctypes.c_int, ctypes.c_void_p
        lib.moe_ref_f64.restype = i
        lib.moe_ref_f64.argtypes = [p, p, p, p, p, p, p, p, i, i, i, i, i, p, i]
        lib.moe_ref_e4m3_decode.restype = ctypes.c_double
        lib.moe_ref_e4m3_decode.argtypes = [ctypes.c_uint8]
        lib.moe_ref_e4m3_encode.restype = ctypes.c_uint8
        lib.moe_ref_e4m3_encode.argtypes = [ctypes.c_float]
        lib.moe_ref_intermediate_f64.restype = i
        lib.moe_ref_intermediate_f64.argtypes = [p, p, p, p, i, i, i, i, i, i]
        lib.moe_ref_down_f64.restype = i
        lib.moe_ref_down_f64.argtypes = [p, p, p, p, p, i, i, i, i]
        lib.moe_ref_quant_group.restype = None
        lib.moe_ref_quant_group.argtypes = [p, p, p]
        _moe_lib = lib
    return _moe_lib


def e4m3_decode(code: int) -> float:
    return float(_load_moe().moe_ref_e4m3_decode(int(code)))


def e4m3_encode(value: float) -> int:
    return int(_load_moe().moe_ref_e4m3_encode(float(np.float32(value))))


def quant_group(v):
    """e4m3 codes [128] and the fp32 scale of one group of 128 fp32 values."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    if v.shape != (128,):
        raise ValueError("a group has 128 values")
    code = np.empty(128, dtype=np.uint8)
    scale = np.empty(1, dtype=np.float32)
    _load_moe().moe_ref_quant_group(_ptr(v), _ptr(code), _ptr(scale))
    return code, float(scale[0])


def moe_ref(x, ids, wts, w13, s13, w2, s2, rows=None):
    """Reference MoE feed-forward output (fp64) for all tokens or the listed ones: [R, H].

    x [T,H] uint16 (bf16 bits); ids [T,KTOP] int32 (local expert or negative); wts [T,KTOP] fp32;
    w13 [E,2I,H] / w2 [E,H,I] uint8 e4m3 codes; s13 [E,2I/128,H/128] / s2 [E,H/128,I/128] fp32.
    """
    lib = _load_moe()
    T, H = x.shape
    E, I2, _ = w13.shape
    I, K = I2 // 2, ids.shape[1]
    if w13.shape != (E, 2 * I, H) or w2.shape != (E, H, I) or ids.shape != (T, K) or wts.shape != (T, K) \
            or s13.shape != (E, 2 * I // 128, H // 128) or s2.shape != (E, H // 128, I // 128):
        raise ValueError("inconsistent MoE shapes")
    x = np.ascontiguousarray(x, dtype=np.uint16)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    wts = np.ascontiguousarray(wts, dtype=np.float32)
    w13, w2 = np.ascontiguousarray(w13, dtype=np.uint8), np.ascontiguousarray(w2, dtype=np.uint8)
    s13, s2 = np.ascontiguousarray(s13, dtype=np.float32), np.ascontiguousarray(s2, dtype=np.float32)
    rows_a = None if rows is None else np.ascontiguousarray(rows, dtype=np.int32)
    R = T if rows_a is None else rows_a.shape[0]
    y = np.empty((R, H), dtype=np.float64)
    rc = lib.moe_ref_f64(_ptr(x), _ptr(ids), _ptr(wts), _ptr(w13), _ptr(s13), _ptr(w2), _ptr(s2), _ptr(y),
                         T, H, I, E, K, _ptr(rows_a) if rows_a is not None else None, R)
    if rc != 0:
        raise RuntimeError("moe_ref failed with code %d" % rc)
    return y


def moe_intermediate(x, w13, s13, t: int, e: int):
    """Steps 1-2 of the MoE reference for token t on local expert e: the gated intermediate a [I] in
    fp64, before it is rounded to fp32 and requantized."""
    T, H = x.shape
    E, I2, _ = w13.shape
    a = np.empty(I2 // 2, dtype=np.float64)
    x = np.ascontiguousarray(x, dtype=np.uint16)
    w13, s13 = np.ascontiguousarray(w13, dtype=np.uint8), np.ascontiguousarray(s13, dtype=np.float32)
    rc = _load_moe().moe_ref_intermediate_f64(_ptr(x), _ptr(w13), _ptr(s13), _ptr(a), T, H, I2 // 2, E, int(t), int(e))
    if rc != 0:
        raise RuntimeError("moe_intermediate failed with code %d" % rc)
    return a


def moe_down(aq, a_scales, w2, s2, e: int):
    """Step 4 alone: the down-projection row o [H] (fp64) of given intermediate codes aq [I] (uint8)
    and group scales [I/128] (fp32) on local expert e."""
    E, H, I = w2.shape
    aq = np.ascontiguousarray(aq, dtype=np.uint8)
    a_scales = np.ascontiguousarray(a_scales, dtype=np.float32)
    if aq.shape != (I,) or a_scales.shape != (I // 128,):
        raise ValueError("aq [I], scales [I/128]")
    w2, s2 = np.ascontiguousarray(w2, dtype=np.uint8), np.ascontiguousarray(s2, dtype=np.float32)
    o = np.empty(H, dtype=np.float64)
    rc = _load_moe().moe_ref_down_f64(_ptr(aq), _ptr(a_scales), _ptr(w2), _ptr(s2), _ptr(o), H, I, E, int(e))
    if rc != 0:
        raise RuntimeError("moe_down failed with code %d" % rc)
    return o
