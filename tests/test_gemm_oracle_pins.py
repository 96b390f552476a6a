"""Pins of the fp64 GEMM reference (oracle/gemm_ref.c) to things other than itself:
a hand-computed example, closed forms, exact integer arithmetic, an independent library
matmul, and invariants chosen so that a dropped term, a transposed operand, a wrong
leading dimension or a wrong layout flag fails at least one of them."""
import os

import numpy as np
import pytest

import oracle
from paper_2604_18616_amd import inputs as I

GOLD = os.path.join(os.path.dirname(__file__), "golden", "gemm_hand_example.txt")


def bits(x):
    """exact bf16 bit patterns of values that are representable in bf16"""
    h = I.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))
    assert np.array_equal(I.bf16_bits_to_f32(h), np.asarray(x, dtype=np.float32)), "test values must be exact in bf16"
    return h


def rnd(shape, seed, sigma=1.0):
    n = int(np.prod(shape))
    return I.f32_to_bf16_bits((I.normal_stream(seed, 0, n) * sigma).astype(np.float32)).reshape(shape)


def f64(h):
    return I.bf16_bits_to_f32(h).astype(np.float64)


def test_hand_example_from_the_definition():
    rows = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        rows[key] = np.array([float(v) for v in vals])
    a, b = bits(rows["A"].reshape(2, 3)), bits(rows["B"].reshape(3, 2))
    c, s = oracle.gemm_ref(a, b)
    assert np.array_equal(c, rows["C"].reshape(2, 2))
    assert np.array_equal(s, rows["S"].reshape(2, 2))
    # the same product with B stored [N,K]
    c_t, s_t = oracle.gemm_ref(a, np.ascontiguousarray(b.T), b_is_nk=True)
    assert np.array_equal(c_t, c) and np.array_equal(s_t, s)


def test_identity_and_permutation_matrices():
    a = rnd((7, 5), 11)
    eye = bits(np.eye(5))
    c, s = oracle.gemm_ref(a, eye)
    assert np.array_equal(c, f64(a)) and np.array_equal(s, np.abs(f64(a)))
    perm = np.array([3, 0, 4, 1, 2])
    p = bits(np.eye(5)[:, perm])          # (A P)[:, j] = A[:, perm[j]]
    c, _ = oracle.gemm_ref(a, p)
    assert np.array_equal(c, f64(a)[:, perm])
    # a transposed-operand mistake would give A^T-shaped or permuted-the-other-way results
    c_t, _ = oracle.gemm_ref(a, p, b_is_nk=True)      # now B^T = P^T: columns go the inverse way
    assert np.array_equal(c_t[:, perm], f64(a))


def test_all_ones_counts_the_inner_dimension():
    for M, N, K in ((3, 4, 1), (2, 2, 257), (5, 1, 1000)):
        c, s = oracle.gemm_ref(bits(np.ones((M, K))), bits(np.ones((K, N))))
        assert np.array_equal(c, np.full((M, N), float(K))) and np.array_equal(s, c)


def test_rank_one_outer_product():
    u, v = rnd((9, 1), 21), rnd((1, 6), 22)
    c, _ = oracle.gemm_ref(u, v)
    assert np.array_equal(c, f64(u) * f64(v))          # one product per entry: exact in fp64


def test_small_integers_match_exact_integer_arithmetic():
    rng = np.random.default_rng(5)
    A = rng.integers(-8, 9, size=(13, 70))
    B = rng.integers(-8, 9, size=(70, 11))
    want = [[sum(int(A[i, k]) * int(B[k, j]) for k in range(70)) for j in range(11)] for i in range(13)]
    c, s = oracle.gemm_ref(bits(A), bits(B))
    assert np.array_equal(c, np.array(want, dtype=np.float64))
    assert np.array_equal(s, (np.abs(A) @ np.abs(B)).astype(np.float64))
    c_t, _ = oracle.gemm_ref(bits(A), bits(B.T.copy()), b_is_nk=True)
    assert np.array_equal(c_t, c)


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (17, 33, 65), (64, 48, 300), (100, 7, 129)])
@pytest.mark.parametrize("b_is_nk", [False, True])
def test_against_library_matmul_with_padded_rows(M, N, K, b_is_nk):
    """numpy's fp64 matmul is an independent second implementation; operands are slices of
    wider arrays, so a wrong leading dimension reads the NaN-free but different padding."""
    a_full, b_full = rnd((M, K + 5), 31 + M), rnd(((N, K + 3) if b_is_nk else (K, N + 9)), 32 + N)
    a = a_full[:, :K]
    b = b_full[:, :K] if b_is_nk else b_full[:, :N]
    c, s = oracle.gemm_ref(a, b, b_is_nk=b_is_nk)
    bm = f64(b).T if b_is_nk else f64(b)
    want = f64(a) @ bm
    bound = 4 * K * np.finfo(np.float64).eps * (np.abs(f64(a)) @ np.abs(bm))
    assert np.all(np.abs(c - want) <= bound)
    assert np.all(np.abs(s - np.abs(f64(a)) @ np.abs(bm)) <= bound)


def test_non_square_shapes_catch_swapped_dimensions():
    a, b = rnd((3, 10), 41), rnd((10, 6), 42)
    c, _ = oracle.gemm_ref(a, b)
    assert c.shape == (3, 6)
    np.testing.assert_allclose(c[2, 5], float(np.dot(f64(a)[2], f64(b)[:, 5])), rtol=1e-13)
    with pytest.raises(ValueError):
        oracle.gemm_ref(a, b, b_is_nk=True)            # [N,K] would need 10 columns


def test_matrix_vector_associativity():
    a, b, x = rnd((12, 40), 51), rnd((40, 9), 52), np.linspace(-1, 1, 9)
    c, _ = oracle.gemm_ref(a, b)
    np.testing.assert_allclose(c @ x, f64(a) @ (f64(b) @ x), rtol=1e-12, atol=1e-12)


def test_block_decomposition_over_k():
    """Summing the products of the two K halves gives the whole product (a dropped or doubled
    term at a block edge breaks it)."""
    a, b = rnd((6, 96), 61), rnd((96, 8), 62)
    c, _ = oracle.gemm_ref(a, b)
    c1, _ = oracle.gemm_ref(a[:, :37], b[:37])
    c2, _ = oracle.gemm_ref(a[:, 37:], b[37:])
    np.testing.assert_allclose(c1 + c2, c, rtol=1e-13, atol=1e-13)


def test_samples_agree_with_the_full_product():
    w = I.GemmWorkload("t", 40, 50, 77, 71)
    a, b = I.make_ab(w)
    c, s = oracle.gemm_ref(a, b)
    si, sj = I.sample_outputs(w, 200)
    assert si.shape == (200,) and si.min() >= 0 and si.max() < 40 and sj.max() < 50
    cs, ss = oracle.gemm_ref_samples(a, b, si, sj)
    assert np.array_equal(cs, c[si, sj]) and np.array_equal(ss, s[si, sj])
    wt = I.GemmWorkload("t", 40, 50, 77, 71, b_is_nk=True)
    at, bt = I.make_ab(wt)
    assert bt.shape == (50, 77)
    ct, _ = oracle.gemm_ref(at, bt, b_is_nk=True)
    cts, _ = oracle.gemm_ref_samples(at, bt, si, sj, b_is_nk=True)
    assert np.array_equal(cts, ct[si, sj])


def test_bad_arguments_are_refused():
    a, b = rnd((4, 8), 81), rnd((8, 4), 82)
    with pytest.raises(ValueError):
        oracle.gemm_ref(a, b[:7])
    with pytest.raises(TypeError):
        oracle.gemm_ref(a.astype(np.float32), b)
    with pytest.raises(RuntimeError):
        oracle.gemm_ref_samples(a, b, [4], [0])         # row index out of range


def test_gemm_workload_table():
    w = I.GEMM_WORKLOADS["G1024"]
    assert (w.M, w.N, w.K, w.b_is_nk) == (1024, 1024, 1024, False) and w.flops() == 2.0 * 1024 ** 3
    assert I.GEMM_WORKLOADS["G16384T"].b_is_nk and I.GEMM_WORKLOADS["G16384T"].bytes() == 6.0 * 16384 ** 2
    a, b = I.make_ab(I.GemmWorkload("s", 64, 32, 48, 9))
    x = np.concatenate([I.bf16_bits_to_f32(a).ravel(), I.bf16_bits_to_f32(b).ravel()])
    assert a.shape == (64, 48) and b.shape == (48, 32) and abs(x.mean()) < 0.1 and abs(x.std() - 1) < 0.1
