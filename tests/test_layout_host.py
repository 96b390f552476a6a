"""Host-side enumeration of the kernels' index maps (csrc/attn_layout.h): operand pairing at
both MFMA sites, staging bijection, bank model, and detection of a planted layout bug."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_layout_invariants(tmp_path):
    exe = str(tmp_path / "layout_check")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-Wall", "-o", exe,
                           os.path.join(ROOT, "tests", "host", "layout_check.cpp")])
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    assert "layout checks passed" in res.stdout


def test_gemm_layout_invariants(tmp_path):
    exe = str(tmp_path / "gemm_layout_check")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-Wall", "-o", exe,
                           os.path.join(ROOT, "tests", "host", "gemm_layout_check.cpp")])
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    assert "gemm layout checks passed" in res.stdout
