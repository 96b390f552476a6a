"""ctypes binding of the C-ABI attention library (argument marshalling only).

Function names mirror include/attn.h.  Tensors are torch CUDA tensors (PyTorch is
used for device memory and streams only); their device pointers and the current
stream handle are passed straight to the library.  There is no fallback: if the
HIP library is missing or fails, the call raises.
"""
from __future__ import annotations

import ctypes
import os

from .build import LIB_PATH, build_library, stale_sources

_lib = None


class AttnError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("attn_fwd failed (%d): %s" % (code, msg))
        self.code = code


def load_library(build_if_missing: bool = True):
    """Load libattn_mi355x.so (building it first only if no built library exists; a library older than its
    sources is loaded as it is, with a warning: rebuild with `python -m paper_2604_18616_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            if not build_if_missing:
                raise FileNotFoundError(LIB_PATH)
            build_library()
        elif stale_sources():
            import warnings
            warnings.warn("libattn_mi355x.so is older than %s: rebuild it" % ", ".join(stale_sources()))
        lib = ctypes.CDLL(LIB_PATH)
        i, f, p = ctypes.c_int, ctypes.c_float, ctypes.c_void_p
        lib.attn_fwd.restype = i
        lib.attn_fwd.argtypes = [p, p, p, p, p, i, i, i, i, i, i, i, f, p]
        lib.attn_fwd_tile.restype = i
        lib.attn_fwd_tile.argtypes = [p, p, p, p, p, i, i, i, i, i, i, i, f, i, p]
        lib.attn_fwd_strided.restype = i
        lib.attn_fwd_strided.argtypes = [p, p, p, p, p, i, i, i, i, i, i, p, p, p, p, i, f, p]
        ll = ctypes.c_longlong
        lib.gemm_bf16.restype = i
        lib.gemm_bf16.argtypes = [p, p, p, i, i, i, ll, ll, ll, i, p]
        lib.gemm_bf16_tile.restype = i
        lib.gemm_bf16_tile.argtypes = [p, p, p, i, i, i, ll, ll, ll, i, i, p]
        lib.gemm_bf16_auto_tile.restype = i
        lib.gemm_bf16_auto_tile.argtypes = [i, i]
        lib.gemm_bf16_flops.restype = ctypes.c_double
        lib.gemm_bf16_flops.argtypes = [i, i, i]
        lib.moe_ffn_fp8_workspace_bytes.restype = ctypes.c_size_t
        lib.moe_ffn_fp8_workspace_bytes.argtypes = [i, i, i, i, i]
        lib.moe_ffn_fp8_workspace_offset.restype = ctypes.c_longlong
        lib.moe_ffn_fp8_workspace_offset.argtypes = [i, i, i, i, i, i]
        lib.moe_ffn_fp8.restype = i
        lib.moe_ffn_fp8.argtypes = [p, p, p, p, p, p, p, p, i, i, i, i, i, p, ctypes.c_size_t, p]
        lib.moe_ffn_fp8_ex.restype = i
        lib.moe_ffn_fp8_ex.argtypes = [p, p, p, p, p, p, p, p, i, i, i, i, i, p, ctypes.c_size_t, i, i, i, p]
        lib.moe_ffn_fp8_static.restype = i
        lib.moe_ffn_fp8_static.argtypes = [p, p, p, p, p, p, p, p, i, i, i, i, i, p]
        lib.moe_ffn_fp8_flops_per_pair.restype = ctypes.c_double
        lib.moe_ffn_fp8_flops_per_pair.argtypes = [i, i]
        lib.attn_strerror.restype = ctypes.c_char_p
        lib.attn_strerror.argtypes = [i]
        lib.attn_version.restype = i
        lib.attn_version.argtypes = []
        lib.attn_fwd_flops.restype = ctypes.c_double
        lib.attn_fwd_flops.argtypes = [i, i, i, i, i, i, i]
        lib.attn_mfma_calibration.restype = ctypes.c_double
        lib.attn_mfma_calibration.argtypes = [p, i, i, p]
        lib.attn_mfma_calibration_data.restype = ctypes.c_double
        lib.attn_mfma_calibration_data.argtypes = [p, i, i, i, p]
        lib.attn_device_info.restype = i
        lib.attn_device_info.argtypes = [i, ctypes.POINTER(i), ctypes.POINTER(i), ctypes.POINTER(ctypes.c_double)]
        _lib = lib
    return _lib


def strerror(code: int) -> str:
    return load_library().attn_strerror(int(code)).decode()


def version() -> int:
    return load_library().attn_version()


def device_info(device: int = 0) -> dict:
    """Compute units, maximum shader clock and the bf16 matrix peak that follows (attn_device_info)."""
    cus, khz, peak = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_double(0.0)
    rc = load_library().attn_device_info(int(device), ctypes.byref(cus), ctypes.byref(khz), ctypes.byref(peak))
    if rc != 0:
        raise AttnError(rc, strerror(rc))
    return {"cus": cus.value, "clock_mhz": khz.value / 1e3, "bf16_peak_tflops_from_props": peak.value}


def attn_fwd_flops(B, Hq, Hkv, Sq, Sk, D, causal) -> float:
    return load_library().attn_fwd_flops(B, Hq, Hkv, Sq, Sk, D, int(bool(causal)))


def attn_fwd_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, Sq, Sk, D, causal, scale, stream_ptr, wg_rows=0) -> int:
    """Direct call with integer device addresses; returns the library's status code.  wg_rows != 0 goes
    through attn_fwd_tile (workgroup shape forced: 128 or 256 query rows)."""
    lib = load_library()
    if wg_rows:
        return lib.attn_fwd_tile(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, Sq, Sk, D,
                                 int(bool(causal)), float(scale), int(wg_rows), stream_ptr)
    return lib.attn_fwd(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, Sq, Sk, D,
                        int(bool(causal)), float(scale), stream_ptr)


def _strides3(t):
    return (ctypes.c_longlong * 3)(t.stride(0), t.stride(1), t.stride(2))


def attn_fwd(q, k, v, o=None, lse=None, causal=False, scale=None, stream=None):
    """O, LSE = attention forward of bf16 CUDA tensors q [B,Hq,Sq,D], k/v [B,Hkv,Sk,D].

    The tensors may be strided views (e.g. a [B,S,H,D] buffer transposed to [B,H,S,D]) as long
    as the last dimension is contiguous; contiguous inputs take attn_fwd, anything else
    attn_fwd_strided.  o (bf16, q's shape) and lse (fp32 [B,Hq,Sq], contiguous) are allocated
    with torch if not given.  The kernel is enqueued on `stream` (default: torch's current
    stream); no sync.
    """
    import torch

    if not (q.is_cuda and k.is_cuda and v.is_cuda):
        raise ValueError("q, k, v must be CUDA tensors: there is no CPU path")
    for t in (q, k, v):
        if t.dtype != torch.bfloat16 or t.dim() != 4 or t.stride(3) != 1:
            raise ValueError("q, k, v must be 4-D bfloat16 tensors with a contiguous last dimension")
    B, Hq, Sq, D = q.shape
    Bk, Hkv, Sk, Dk = k.shape
    if v.shape != k.shape or Bk != B or Dk != D:
        raise ValueError("inconsistent q/k/v shapes")
    if o is None:
        o = torch.empty_like(q)          # keeps q's layout for dense views
    if o.shape != q.shape or o.dtype != torch.bfloat16 or o.stride(3) != 1:
        raise ValueError("o must be bfloat16 with q's shape and a contiguous last dimension")
    if lse is None:
        lse = torch.empty((B, Hq, Sq), dtype=torch.float32, device=q.device)
    if not lse.is_cuda or lse.dtype != torch.float32 or tuple(lse.shape) != (B, Hq, Sq) or not lse.is_contiguous():
        raise ValueError("lse must be a contiguous float32 CUDA tensor of shape [B, Hq, Sq]")
    if not o.is_cuda or any(t.device != q.device for t in (k, v, o, lse)):
        raise ValueError("q, k, v, o, lse must live on one CUDA device")
    if scale is None:
        scale = float(D) ** -0.5
    if stream is None:
        stream = torch.cuda.current_stream(q.device)
    lib = load_library()
    if all(t.is_contiguous() for t in (q, k, v, o)):
        rc = lib.attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                          B, Hq, Hkv, Sq, Sk, D, int(bool(causal)), float(scale), stream.cuda_stream)
    else:
        rc = lib.attn_fwd_strided(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                                  B, Hq, Hkv, Sq, Sk, D, _strides3(q), _strides3(k), _strides3(v), _strides3(o),
                                  int(bool(causal)), float(scale), stream.cuda_stream)
    if rc != 0:
        raise AttnError(rc, strerror(rc))
    return o, lse


def gemm_bf16(a, b, c=None, b_is_nk=False, stream=None, tile=0):
    """C = A B for bf16 CUDA tensors a [M,K] and b [K,N] (or [N,K] if b_is_nk); rows contiguous,
    row pitch free.  c (bf16 [M,N]) is allocated with torch if not given.  Enqueued on `stream`
    (default: torch's current stream); no sync.  tile: 0 (by size) or a shape code of gemm.h: 64, 128, 1284, 256, 2564, those with 16 appended, or 19216 (gemm_bf16_tile)."""
    import torch

    if not (a.is_cuda and b.is_cuda):
        raise ValueError("a, b must be CUDA tensors: there is no CPU path")
    for t in (a, b):
        if t.dtype != torch.bfloat16 or t.dim() != 2 or t.stride(1) != 1:
            raise ValueError("a, b must be 2-D bfloat16 tensors with contiguous rows")
    M, K = a.shape
    N = b.shape[0] if b_is_nk else b.shape[1]
    if (b.shape[1] if b_is_nk else b.shape[0]) != K:
        raise ValueError("inner dimensions differ")
    if c is None:
        c = torch.empty((M, N), dtype=torch.bfloat16, device=a.device)
    if c.shape != (M, N) or c.dtype != torch.bfloat16 or c.stride(1) != 1:
        raise ValueError("c must be bfloat16 [M,N] with contiguous rows")
    if stream is None:
        stream = torch.cuda.current_stream(a.device)
    rc = load_library().gemm_bf16_tile(a.data_ptr(), b.data_ptr(), c.data_ptr(), M, N, K,
                                       a.stride(0), b.stride(0), c.stride(0), int(bool(b_is_nk)), int(tile), stream.cuda_stream)
    if rc != 0:
        raise AttnError(rc, strerror(rc))
    return c


def moe_workspace_bytes(T, H, I, E, KTOP) -> int:
    return int(load_library().moe_ffn_fp8_workspace_bytes(T, H, I, E, KTOP))


def moe_workspace_offset(T, H, I, E, KTOP, part: int) -> int:
    return int(load_library().moe_ffn_fp8_workspace_offset(T, H, I, E, KTOP, part))


def moe_ffn_fp8(x, ids, wts, w13, s13, w2, s2, y=None, workspace=None, stream=None, row_tile=0):
    """Block-quantized FP8 MoE feed-forward of CUDA tensors: x bf16 [T,H]; ids int32 [T,KTOP] (local
    expert or negative); wts fp32 [T,KTOP]; w13 uint8 [E,2I,H] and w2 uint8 [E,H,I] (e4m3 codes);
    s13 fp32 [E,2I/128,H/128]; s2 fp32 [E,H/128,I/128].  y (bf16 [T,H]) and the workspace (uint8, at
    least moe_workspace_bytes(...)) are allocated with torch if not given.  Enqueued on `stream`
    (default: torch's current stream); no sync.  row_tile: 0 (the default, 128) or 64 (moe_ffn_fp8_ex)."""
    import torch

    for t in (x, ids, wts, w13, s13, w2, s2):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("all MoE tensors must be contiguous CUDA tensors: there is no CPU path")
    T, H = x.shape
    E, I2, _ = w13.shape
    I, K = I2 // 2, ids.shape[1]
    if (x.dtype != torch.bfloat16 or ids.dtype != torch.int32 or wts.dtype != torch.float32 or w13.dtype != torch.uint8
            or w2.dtype != torch.uint8 or s13.dtype != torch.float32 or s2.dtype != torch.float32):
        raise ValueError("dtypes: x bf16, ids int32, wts/s13/s2 fp32, w13/w2 uint8")
    if (w13.shape != (E, 2 * I, H) or w2.shape != (E, H, I) or ids.shape != (T, K) or wts.shape != (T, K)
            or s13.shape != (E, 2 * I // 128, H // 128) or s2.shape != (E, H // 128, I // 128)):
        raise ValueError("inconsistent MoE shapes")
    lib = load_library()
    need = lib.moe_ffn_fp8_workspace_bytes(T, H, I, E, K)
    if y is None:
        y = torch.empty((T, H), dtype=torch.bfloat16, device=x.device)
    if not y.is_cuda or y.dtype != torch.bfloat16 or tuple(y.shape) != (T, H) or not y.is_contiguous():
        raise ValueError("y must be a contiguous bfloat16 CUDA tensor of shape [T, H]")
    current = torch.cuda.current_stream(x.device)
    if stream is None:
        stream = current
    if workspace is None:
        # a temporary is only safe on the stream torch will reuse its memory on: the kernels are still queued
        # when this function returns
        if stream.cuda_stream != current.cuda_stream:
            raise ValueError("pass a workspace when `stream` is not torch's current stream")
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    if (not workspace.is_cuda or workspace.dtype != torch.uint8 or not workspace.is_contiguous()
            or workspace.numel() < need or workspace.data_ptr() % 256):
        raise ValueError("workspace must be a contiguous uint8 CUDA tensor of at least moe_workspace_bytes(...) bytes, 256-byte aligned")
    rc = lib.moe_ffn_fp8_ex(x.data_ptr(), ids.data_ptr(), wts.data_ptr(), w13.data_ptr(), s13.data_ptr(), w2.data_ptr(),
                            s2.data_ptr(), y.data_ptr(), T, H, I, E, K, workspace.data_ptr(), workspace.numel(),
                            0, 4, int(row_tile), stream.cuda_stream)
    if rc != 0:
        raise AttnError(rc, strerror(rc))
    return y
