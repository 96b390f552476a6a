"""MI355X-native flash-attention forward, bf16 GEMM and FP8 MoE feed-forward: HIP kernels behind a C ABI plus a thin binding.

``attn_fwd``, ``gemm_bf16`` and ``moe_ffn_fp8`` (from :mod:`.binding`) marshal device pointers into the C-ABI
library built from ``csrc/``; every step of the computation runs in the HIP kernels.
:mod:`.inputs` generates the seeded synthetic workloads.
"""

__all__ = ["attn_fwd", "gemm_bf16", "moe_ffn_fp8", "load_library", "build_library", "inputs"]


def __getattr__(name):
    if name in ("attn_fwd", "gemm_bf16", "moe_ffn_fp8", "moe_workspace_bytes", "load_library", "attn_fwd_flops", "strerror", "version", "AttnError"):
        from . import binding
        return getattr(binding, name)
    if name == "build_library":
        from .build import build_library
        return build_library
    raise AttributeError(name)
