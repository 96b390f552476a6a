"""MI355X-native flash-attention forward and bf16 GEMM: HIP kernels behind a C ABI plus a thin binding.

``attn_fwd`` and ``gemm_bf16`` (from :mod:`.binding`) marshal device pointers into the C-ABI
library built from ``csrc/``; every step of the computation runs in the HIP kernels.
:mod:`.inputs` generates the seeded synthetic workloads.
"""

__all__ = ["attn_fwd", "gemm_bf16", "load_library", "build_library", "inputs"]


def __getattr__(name):
    if name in ("attn_fwd", "gemm_bf16", "load_library", "attn_fwd_flops", "strerror", "version", "AttnError"):
        from . import binding
        return getattr(binding, name)
    if name == "build_library":
        from .build import build_library
        return build_library
    raise AttributeError(name)
