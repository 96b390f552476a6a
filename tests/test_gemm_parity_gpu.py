"""GPU parity of gemm_bf16 (through the C ABI) against the fp64 reference.

Tolerance (derived from the arithmetic): the kernel accumulates exact bf16 x bf16 products
in fp32 -- one rounding per MFMA step of 16 products, K/16 steps, each at most 2^-24
relative to the running magnitude, which the absolute sum S = sum_k |a_ik||b_kj| bounds --
and rounds the result once to bf16 (relative 2^-9 to nearest, 2^-8 with margin for a
value pushed over a rounding boundary by the accumulation error):
    |c - ref| <= 2^-8 |ref| + (K/16 + 4) 2^-23 S
"""
import numpy as np
import pytest

import oracle
from paper_2604_18616_amd import inputs as I

pytestmark = pytest.mark.gpu


def tol(ref, s, K):
    return 2.0 ** -8 * np.abs(ref) + (K / 16 + 4) * 2.0 ** -23 * s


def dev(bits):
    import torch
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()


def host(t):
    import torch
    return I.bf16_bits_to_f32(t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)


def run(a_bits, b_bits, b_is_nk, pad=(0, 0, 0), shift=0, tile=0):
    """gemm_bf16 on device copies; pad = extra columns in the storage of (a, b, c) so that the
    pitches exceed the rows; shift = element offset of every pointer (alignment cases).  C starts
    as NaN, and the padding of C must stay NaN."""
    import torch
    from paper_2604_18616_amd import binding

    def place(bits, extra):
        r, c = bits.shape
        buf = torch.zeros(r * (c + extra) + shift + 8, dtype=torch.bfloat16, device="cuda")
        view = buf[shift:shift + r * (c + extra)].view(r, c + extra)[:, :c]
        view.copy_(dev(bits))
        return view

    a, b = place(a_bits, pad[0]), place(b_bits, pad[1])
    M, K = a_bits.shape
    N = b_bits.shape[0] if b_is_nk else b_bits.shape[1]
    cbuf = torch.full((M * (N + pad[2]) + shift + 8,), float("nan"), dtype=torch.bfloat16, device="cuda")
    cfull = cbuf[shift:shift + M * (N + pad[2])].view(M, N + pad[2])
    binding.gemm_bf16(a, b, cfull[:, :N], b_is_nk=b_is_nk, tile=tile)
    torch.cuda.synchronize()
    if pad[2]:
        assert torch.isnan(cfull[:, N:].float()).all(), "C padding was written"
    assert torch.isnan(cbuf[:shift].float()).all() and torch.isnan(cbuf[shift + M * (N + pad[2]):].float()).all()
    return host(cfull[:, :N])


def check_full(M, N, K, b_is_nk, seed, pad=(0, 0, 0), shift=0, tile=0):
    w = I.GemmWorkload("t", M, N, K, seed, b_is_nk=b_is_nk)
    a, b = I.make_ab(w)
    print("gemm case M=%d N=%d K=%d nk=%d pad=%s shift=%d tile=%d" % (M, N, K, b_is_nk, pad, shift, tile), flush=True)
    c = run(a, b, b_is_nk, pad, shift, tile)
    ref, s = oracle.gemm_ref(a, b, b_is_nk=b_is_nk)
    assert np.isfinite(c).all()
    err = np.abs(c - ref)
    bad = err > tol(ref, s, K)
    assert not bad.any(), ("%d of %d outputs off, worst %g at %s" % (bad.sum(), bad.size, err.max(), np.argwhere(bad)[:4].tolist()))


# tiled kernel: whole tiles, several tiles, ragged M / N (multiples of 8), K tails (multiples of 8)
TILED = [(256, 256, 32), (256, 256, 64), (256, 256, 96), (256, 256, 128), (256, 256, 160), (512, 256, 192), (256, 768, 320), (300, 264, 200), (100, 40, 72),
         (1, 8, 8), (257, 8, 24), (8, 520, 136), (513, 512, 64)]


@pytest.mark.parametrize("tile", [64, 128, 1284, 256, 2564, 25616, 256416, 12816, 128416, 6416, 19216])
@pytest.mark.parametrize("b_is_nk", [False, True])
@pytest.mark.parametrize("M,N,K", TILED)
def test_tiled_kernel_small_shapes(M, N, K, b_is_nk, tile):
    check_full(M, N, K, b_is_nk, seed=100 + M + N + K, tile=tile)


@pytest.mark.parametrize("tile", [64, 128, 1284, 256, 2564, 25616, 256416, 12816, 128416, 6416, 19216])
@pytest.mark.parametrize("b_is_nk", [False, True])
def test_tiled_kernel_padded_pitches(b_is_nk, tile):
    check_full(264, 272, 200, b_is_nk, seed=7, pad=(8, 16, 24), tile=tile)


# general kernel: sizes, pitches or addresses the 16-byte pieces of the tiled kernel cannot take
@pytest.mark.parametrize("b_is_nk", [False, True])
@pytest.mark.parametrize("M,N,K,pad,shift", [(33, 17, 5, (0, 0, 0), 0), (64, 64, 16, (0, 0, 0), 1), (70, 130, 37, (3, 5, 1), 0),
                                             (1, 1, 1, (0, 0, 0), 0), (128, 72, 64, (0, 0, 0), 3)])
def test_general_kernel(M, N, K, pad, shift, b_is_nk):
    check_full(M, N, K, b_is_nk, seed=300 + M + N + K, pad=pad, shift=shift)


def test_exact_small_integers():
    """Products and sums of small integers are exact in fp32 and (here) in bf16: bit-exact result."""
    rng = np.random.default_rng(3)
    A = rng.integers(-3, 4, size=(256, 128)).astype(np.float32)
    B = rng.integers(-3, 4, size=(128, 256)).astype(np.float32)
    want = A.astype(np.float64) @ B.astype(np.float64)
    assert np.abs(want).max() <= 256                   # integers up to 256 are exact in bf16
    for tile in (64, 128, 1284, 256, 2564, 25616, 256416, 12816, 128416, 6416, 19216):
        assert np.array_equal(run(I.f32_to_bf16_bits(A), I.f32_to_bf16_bits(B), False, tile=tile), want)


@pytest.mark.parametrize("name,tile", [("G1024", 0), ("G1024T", 256), ("G2048", 0), ("G2048T", 0), ("G4096", 0), ("G4096T", 128), ("G4096", 2564), ("G2048T", 2564),
                                       ("G8192", 0), ("G8192T", 0), ("G16384", 0), ("G16384T", 0)])
def test_paper_sizes_on_sampled_outputs(name, tile):
    w = I.GEMM_WORKLOADS[name]
    a, b = I.make_ab(w)
    print("gemm workload", name, "tile", tile, flush=True)
    c = run(a, b, w.b_is_nk, tile=tile)
    si, sj = I.sample_outputs(w, 4096)
    ref, s = oracle.gemm_ref_samples(a, b, si, sj, b_is_nk=w.b_is_nk)
    err = np.abs(c[si, sj] - ref)
    bad = err > tol(ref, s, w.K)
    assert np.isfinite(c).all() and not bad.any(), (name, int(bad.sum()), float(err.max()))
