"""Build the C-ABI library (attention forward, bf16 GEMM, FP8 MoE) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
OBJ_DIR = os.path.join(_HERE, "_build")
LIB_PATH = os.path.join(_HERE, "libattn_mi355x.so")
SOURCES = ["attn_api.cpp", "attn_fwd_kernel.hip", "gemm_api.cpp", "gemm_bf16_kernel.hip",
           "moe_api.cpp", "moe_fp8_kernel.hip"]
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 instructions are kept out of all device code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the device-only target feature and says so: harmless
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out, flush=True)


def _newest_header() -> float:
    dirs = (CSRC, os.path.join(os.path.dirname(_HERE), "include"))
    return max(os.path.getmtime(os.path.join(d, f)) for d in dirs for f in os.listdir(d) if f.endswith(".h"))


def stale_sources() -> list:
    """Sources and headers that are newer than the built library (empty if there is none to compare with)."""
    if not os.path.exists(LIB_PATH):
        return []
    t = os.path.getmtime(LIB_PATH)
    dirs = (CSRC, os.path.join(os.path.dirname(_HERE), "include"))
    return sorted(f for d in dirs for f in os.listdir(d) if os.path.getmtime(os.path.join(d, f)) > t)


def build_library(verbose: bool = False, incremental: bool = False) -> str:
    """Compile every source under csrc/ (one hipcc per file, in parallel) and link libattn_mi355x.so.
    Always recompiles unless `incremental`, which keeps the objects that are newer than their source
    and than every header."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc, hdr = hipcc_path(), _newest_header()
    objs, jobs = [], []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ_DIR, s + ".o")
        objs.append(obj)
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), hdr):
            continue
        jobs.append([hipcc, *HIPCC_FLAGS, "-c", "-o", obj, src])
    with ThreadPoolExecutor(max(1, min(len(jobs), os.cpu_count() or 1))) as ex:
        list(ex.map(lambda c: _run(c, verbose), jobs))
    tmp = LIB_PATH + ".tmp.%d" % os.getpid()
    try:
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs], verbose)
    except RuntimeError:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True, incremental="--incremental" in sys.argv))
