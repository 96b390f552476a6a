"""The C-ABI library: it loads, exports every symbol include/attn.h declares, and every
argument error is reported before any HIP call (so these run on a machine with no GPU)."""
import ctypes
import math
import os
import re

import pytest

from paper_2604_18616_amd import binding
from paper_2604_18616_amd.inputs import WORKLOADS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "attn.h")


@pytest.fixture(scope="module")
def lib():
    return binding.load_library()       # builds only if no built library is present


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return re.findall(r"\b([a-z_][a-z0-9_]*)\s*\([^;{]*\)\s*;", src)


def test_header_declares_the_boundary():
    names = declared_functions()
    assert set(names) == {"attn_fwd", "attn_strerror", "attn_version", "attn_fwd_flops", "attn_mfma_calibration", "attn_mfma_calibration_data", "attn_fwd_strided", "attn_device_info", "attn_fwd_tile"}


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name
    assert lib.attn_version() >= 100


def test_error_codes_match_header(lib):
    src = open(HEADER).read()
    codes = {m.group(1): int(m.group(2)) for m in re.finditer(r"(ATTN_[A-Z_]+)\s*=\s*(-?\d+)", src)}
    assert codes["ATTN_OK"] == 0 and len(codes) == 8
    msgs = {c: lib.attn_strerror(c).decode() for c in codes.values()}
    assert len(set(msgs.values())) == len(msgs)            # distinct, non-empty messages
    assert all(msgs.values())
    assert "unknown" in lib.attn_strerror(-99).decode()


A16 = 0x1000   # fake, aligned, never dereferenced: validation returns before any HIP call


def call(lib, q=A16, k=A16, v=A16, o=A16, lse=A16, B=1, Hq=4, Hkv=2, Sq=128, Sk=128, D=128, causal=1, scale=0.1):
    return lib.attn_fwd(q, k, v, o, lse, B, Hq, Hkv, Sq, Sk, D, causal, scale, None)


def test_argument_errors_are_reported_without_a_gpu(lib):
    assert call(lib, q=None) == -1 and call(lib, k=None) == -1 and call(lib, v=None) == -1 and call(lib, o=None) == -1
    for kw in (dict(B=0), dict(Hq=0), dict(Hkv=0), dict(Sq=0), dict(Sk=-3), dict(D=0), dict(Hq=5, Hkv=2)):
        assert call(lib, **kw) == -2, kw
    assert call(lib, B=1 << 20, Hq=1 << 10, Hkv=1, Sq=1 << 20) == -2           # grid overflow
    for D in (32, 96, 256, 80):
        assert call(lib, D=D) == -3
    for kw in (dict(q=A16 + 2), dict(k=A16 + 8), dict(v=A16 + 4), dict(o=A16 + 1), dict(lse=A16 + 2)):
        assert call(lib, **kw) == -4, kw
    for s in (0.0, -0.5, math.nan, math.inf, -math.inf):
        assert call(lib, scale=s) == -5, s


def test_tile_entry_point_argument_errors(lib):
    t = lambda rows, q=A16, D=128: lib.attn_fwd_tile(q, A16, A16, A16, A16, 1, 4, 2, 128, 128, D, 1, 0.1, rows, None)
    for rows in (1, 64, 129, 512, -128):
        assert t(rows) == -3, rows                         # only 0, 128, 256 name a workgroup shape
    assert t(128, q=None) == -1 and t(256, D=96) == -3 and t(0, q=A16 + 2) == -4


def test_strided_entry_point_argument_errors(lib):
    L3 = ctypes.c_longlong * 3
    good_q, good_k = L3(4 * 128 * 128, 128 * 128, 128), L3(2 * 128 * 128, 128 * 128, 128)

    def scall(qs=good_q, ks=good_k, vs=good_k, os_=good_q, **kw):
        a = dict(q=A16, k=A16, v=A16, o=A16, lse=A16, B=1, Hq=4, Hkv=2, Sq=128, Sk=128, D=128, causal=1, scale=0.1)
        a.update(kw)
        return lib.attn_fwd_strided(a["q"], a["k"], a["v"], a["o"], a["lse"], a["B"], a["Hq"], a["Hkv"], a["Sq"], a["Sk"],
                                    a["D"], qs, ks, vs, os_, a["causal"], a["scale"], None)

    assert scall(qs=None) == -1 and scall(os_=None) == -1 and scall(q=None) == -1
    assert scall(qs=L3(0, 128 * 128, 64)) == -2            # row stride smaller than D: rows overlap
    assert scall(ks=L3(-8, 128 * 128, 128)) == -2
    assert scall(vs=L3(0, 128 * 128, 1 << 28)) == -2
    assert scall(qs=L3(4 * 128 * 128, 128 * 128, 132)) == -4   # not a multiple of 8 elements
    assert scall(os_=L3(4, 128 * 128, 128)) == -4
    assert scall(D=96) == -3 and scall(scale=0.0) == -5 and scall(Hq=3) == -2


def test_flops_helper_matches_workload_table(lib):
    for w in WORKLOADS.values():
        assert lib.attn_fwd_flops(w.B, w.Hq, w.Hkv, w.Sq, w.Sk, w.D, int(w.causal)) == w.flops()
    assert lib.attn_fwd_flops(1, 1, 1, 3, 5, 64, 1) == 4 * 64 * (3 + 4 + 5)     # bottom-right aligned
    assert lib.attn_fwd_flops(1, 1, 1, 5, 3, 64, 1) == 4 * 64 * (0 + 0 + 1 + 2 + 3)
    assert lib.attn_fwd_flops(1, 3, 2, 4, 4, 64, 0) == -1.0


def test_calibration_rejects_bad_arguments_without_a_gpu(lib):
    assert lib.attn_mfma_calibration(None, 256, 10, None) == -1.0
    assert lib.attn_mfma_calibration(A16, 0, 10, None) == -1.0
    assert lib.attn_mfma_calibration(A16, 256, 0, None) == -1.0
    assert lib.attn_mfma_calibration_data(None, 256, 10, 2, None) == -1.0
    assert lib.attn_mfma_calibration_data(A16, 256, 10, 6, None) == -1.0
    assert lib.attn_mfma_calibration_data(A16, 256, 10, -1, None) == -1.0


def test_python_binding_refuses_cpu_tensors():
    torch = pytest.importorskip("torch")
    q = torch.zeros(1, 2, 8, 64, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        binding.attn_fwd(q, q, q)


# ---------------------------------------------------------------------------------------------
# gemm.h
# ---------------------------------------------------------------------------------------------
GEMM_HEADER = os.path.join(ROOT, "include", "gemm.h")


def test_gemm_header_symbols_are_exported(lib):
    src = re.sub(r"/\*.*?\*/", "", open(GEMM_HEADER).read(), flags=re.S)
    names = re.findall(r"\b([a-z_][a-z0-9_]*)\s*\([^;{]*\)\s*;", src)
    assert set(names) == {"gemm_bf16", "gemm_bf16_tile", "gemm_bf16_auto_tile", "gemm_bf16_flops"}
    for name in names:
        assert hasattr(lib, name), name
    assert lib.gemm_bf16_flops(1024, 512, 256) == 2.0 * 1024 * 512 * 256
    assert lib.gemm_bf16_flops(0, 5, 5) == 0.0
    # the tile rule at the paper's square sizes and at the cross-overs it was measured on
    lib.gemm_bf16_auto_tile.restype = ctypes.c_int
    lib.gemm_bf16_auto_tile.argtypes = [ctypes.c_int, ctypes.c_int]
    want = {1024: 64, 1280: 64, 1536: 1284, 2048: 1284, 2304: 128, 2560: 128, 2816: 128, 3072: 19216, 3328: 19216, 3584: 25616, 3840: 25616,
            4096: 25616, 4608: 19216, 5120: 25616, 6144: 19216, 7168: 25616, 8192: 25616, 16384: 25616}
    assert {s: lib.gemm_bf16_auto_tile(s, s) for s in want} == want
    rect = {(1024, 8192): 128, (8192, 1024): 128, (2048, 4096): 128, (1024, 4096): 1284, (1536, 8192): 19216, (3072, 8192): 19216, (6144, 4096): 19216, (3000, 5000): 25616,
            (1024, 16384): 25616, (256, 16384): 1284, (128, 4096): 64, (64, 1 << 20): 64}
    assert {mn: lib.gemm_bf16_auto_tile(*mn) for mn in rect} == rect
    assert lib.gemm_bf16_auto_tile(0, 8) == 0


def test_gemm_argument_errors_are_reported_without_a_gpu(lib):
    def g(a=A16, b=A16, c=A16, M=256, N=256, K=64, lda=64, ldb=256, ldc=256, nk=0):
        return lib.gemm_bf16(a, b, c, M, N, K, lda, ldb, ldc, nk, None)

    assert g(a=None) == -1 and g(b=None) == -1 and g(c=None) == -1
    for kw in (dict(M=0), dict(N=-1), dict(K=0)):
        assert g(**kw) == -2, kw
    assert g(lda=63) == -2 and g(ldb=255) == -2 and g(ldc=255) == -2
    assert g(nk=1, ldb=63) == -2                      # B stored [N,K]: the pitch must cover K
    assert g(lda=1 << 31) == -2
    assert g(M=(1 << 31) - 1, N=(1 << 31) - 1, ldb=(1 << 31) - 1, ldc=(1 << 31) - 1) == -2   # too many tiles
    assert g(a=A16 + 1) == -4 and g(c=A16 + 3) == -4  # odd addresses cannot hold bf16
    assert lib.gemm_bf16_tile(A16, A16, A16, 256, 256, 64, 64, 256, 256, 0, 96, None) == -3   # tile must be one of the shape codes of gemm.h
    assert lib.gemm_bf16_tile(None, A16, A16, 256, 256, 64, 64, 256, 256, 0, 128, None) == -1


# ---------------------------------------------------------------------------------------------
# moe.h
# ---------------------------------------------------------------------------------------------
MOE_HEADER = os.path.join(ROOT, "include", "moe.h")


def test_moe_header_symbols_are_exported(lib):
    src = re.sub(r"/\*.*?\*/", "", open(MOE_HEADER).read(), flags=re.S)
    names = re.findall(r"\b([a-z_][a-z0-9_]*)\s*\([^;{]*\)\s*;", src)
    assert set(names) == {"moe_ffn_fp8", "moe_ffn_fp8_workspace_bytes", "moe_ffn_fp8_workspace_offset", "moe_ffn_fp8_flops_per_pair",
                          "moe_ffn_fp8_ex", "moe_ffn_fp8_row_tiles", "moe_ffn_fp8_static"}
    for name in names:
        assert hasattr(lib, name), name
    assert lib.moe_ffn_fp8_flops_per_pair(7168, 2048) == 6.0 * 7168 * 2048
    # the row-tile rule: whole tiles and a remainder, one tile for an expert with up to 32 rows more than a tile
    rt = lib.moe_ffn_fp8_row_tiles
    rt.restype = ctypes.c_int
    rt.argtypes = [ctypes.c_int, ctypes.c_int]
    want128 = {0: 0, 1: 1, 64: 1, 128: 1, 129: 1, 160: 1, 161: 2, 256: 2, 257: 3, 288: 3, 289: 3, 700: 6}
    assert {r: rt(r, 0) for r in want128} == want128 and {r: rt(r, 128) for r in want128} == want128
    want64 = {0: 0, 64: 1, 65: 1, 96: 1, 97: 2, 128: 2, 129: 3, 700: 11}
    assert {r: rt(r, 64) for r in want64} == want64
    assert rt(-1, 0) == -1 and rt(10, 32) == -1 and rt(10, 256) == -1
    for r in range(0, 2000, 7):                      # every row lands in exactly one tile of at most row_tile + 32 rows
        for bm in (64, 128):
            n = rt(r, bm)
            assert (n == 0) == (r == 0) and (n - 1) * bm < r <= (n - 1) * bm + bm + 32 if n else True


def test_moe_workspace_size_and_argument_errors(lib):
    need = lib.moe_ffn_fp8_workspace_bytes(1024, 7168, 2048, 32, 4)
    slots = 1024 * 4
    assert need >= slots * 7168 * 4 + slots * 2048 + 1024 * 7168 and need % 256 == 0     # rows, codes of both activations
    assert lib.moe_ffn_fp8_workspace_bytes(1024, 7168 + 64, 2048, 32, 4) == 0            # H not a multiple of 128
    assert lib.moe_ffn_fp8_workspace_bytes(1 << 19, 7168, 2048, 32, 4) == 0              # too many slots
    offs = [lib.moe_ffn_fp8_workspace_offset(1024, 7168, 2048, 32, 4, part) for part in range(13)]
    assert offs[0] == 0 and all(b > a and b % 256 == 0 for a, b in zip(offs, offs[1:])) and offs[12] + slots * 7168 * 4 <= need
    assert lib.moe_ffn_fp8_workspace_offset(1024, 7168, 2048, 32, 4, 13) == -1 and lib.moe_ffn_fp8_workspace_offset(0, 7168, 2048, 32, 4, 0) == -1

    def m(x=A16, ids=A16, wts=A16, w13=A16, s13=A16, w2=A16, s2=A16, y=A16, T=64, H=256, I=128, E=4, K=2, ws=A16, wsb=1 << 30):
        return lib.moe_ffn_fp8(x, ids, wts, w13, s13, w2, s2, y, T, H, I, E, K, ws, wsb, None)

    for name in ("x", "ids", "wts", "w13", "s13", "w2", "s2", "y", "ws"):
        assert m(**{name: None}) == -1, name
    for kw in (dict(T=0), dict(H=100), dict(I=0), dict(E=0), dict(E=257), dict(K=17), dict(H=16384 + 128), dict(wsb=1024)):
        assert m(**kw) == -2, kw
    assert m(x=A16 + 2) == -4 and m(ws=A16 + 16) == -4 and m(ids=A16 + 1) == -4
    # the allocation-free variant: same checks, and sizes beyond the library-owned scratch are refused before any HIP call
    st = lambda T=64, H=256, x=A16, y=A16: lib.moe_ffn_fp8_static(x, A16, A16, A16, A16, A16, A16, y, T, H, 128, 4, 2, None)
    assert st(x=None) == -1 and st(y=None) == -1 and st(T=0) == -2 and st(H=100) == -2
    limit = int(re.search(r"MOE_FFN_FP8_STATIC_MAX_BYTES\s*\((\d+)u\s*<<\s*(\d+)\)", open(MOE_HEADER).read()).expand(r"\1 \2").split()[0]) << 20
    assert limit == 128 << 20
    assert lib.moe_ffn_fp8_workspace_bytes(1024, 7168, 2048, 32, 4) <= limit < lib.moe_ffn_fp8_workspace_bytes(1032, 7168, 2048, 32, 4)
    assert lib.moe_ffn_fp8_static(A16, A16, A16, A16, A16, A16, A16, A16, 1032, 7168, 2048, 32, 4, None) == -7
    assert "scratch" in lib.attn_strerror(-7).decode()
    ex = lambda a, b, rt=0: lib.moe_ffn_fp8_ex(A16, A16, A16, A16, A16, A16, A16, A16, 64, 256, 128, 4, 2, A16, 1 << 30, a, b, rt, None)
    assert ex(-1, 4) == -3 and ex(0, 5) == -3 and ex(3, 2) == -3 and ex(0, 4, 32) == -3 and ex(0, 4, 256) == -3


# ---------------------------------------------------------------------------------------------
# the headers are plain C: a C99 translation unit that includes all three and takes the address of
# every entry point compiles without warnings and links against the library
# ---------------------------------------------------------------------------------------------
def test_headers_are_plain_c_and_link(tmp_path):
    import subprocess
    inc = os.path.join(ROOT, "include")
    protos = {}
    for h in ("attn.h", "gemm.h", "moe.h"):
        src = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, h)).read(), flags=re.S)
        protos[h] = re.findall(r"\b([a-z_][a-z0-9_]*)\s*\([^;{]*\)\s*;", src)
    c = tmp_path / "use_abi.c"
    lines = ['#include "attn.h"', '#include "gemm.h"', '#include "moe.h"', "#include <stdio.h>", "int main(void) {",
             "    const void *fns[] = {"]
    lines += ["        (const void *)%s," % name for h in protos for name in protos[h]]
    lines += ["    };", '    printf("%d entry points, version %d, %s\\n", (int)(sizeof fns / sizeof fns[0]), attn_version(), attn_strerror(0));',
              "    return gemm_bf16_flops(2, 3, 4) == 48.0 && moe_ffn_fp8_row_tiles(150, 0) == 1 ? 0 : 1;", "}"]
    c.write_text("\n".join(lines) + "\n")
    from paper_2604_18616_amd.build import LIB_PATH as lib
    binding.load_library()                       # builds the library first if no built one exists
    exe = str(tmp_path / "use_abi")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", inc, str(c), "-o", exe, lib,
                           "-Wl,-rpath," + os.path.dirname(lib), "-Wl,-rpath,/opt/rocm/lib"])
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    assert "entry points" in res.stdout and "success" in res.stdout
