"""Seeded input generator: determinism, bf16 rounding, distribution, row sampling."""
import numpy as np

from paper_2604_18616_amd import inputs as I


def test_bf16_round_to_nearest_even():
    # 1 + 2^-8 is exactly half way between bf16 neighbours 1 and 1 + 2^-7: ties go to even (1.0)
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 3 * 2.0 ** -8, -2.5, 0.0], np.float32)
    b = I.f32_to_bf16_bits(x)
    back = I.bf16_bits_to_f32(b)
    np.testing.assert_array_equal(back, np.array([1.0, 1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -6, -2.5, 0.0], np.float32))
    # every bf16 value survives a round trip
    allb = np.arange(0, 0x7F80, dtype=np.uint16)
    np.testing.assert_array_equal(I.f32_to_bf16_bits(I.bf16_bits_to_f32(allb)), allb)


def test_bf16_matches_torch_rounding():
    import torch
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * 3
    ours = I.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(ours, ref)


def test_splitmix64_known_values():
    # first outputs of splitmix64 seeded with 0 (published reference sequence of the algorithm)
    r = I.splitmix64(np.arange(3, dtype=np.uint64), 0)
    assert [int(x) for x in r] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_streams_are_deterministic_and_position_addressed():
    a = I.normal_stream(7, 0, 1000)
    b = I.normal_stream(7, 0, 1000)
    c = I.normal_stream(7, 500, 500)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(a[500:], c)
    assert not np.array_equal(a, I.normal_stream(8, 0, 1000))


def test_normal_moments():
    x = I.normal_stream(11, 0, 400000)
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01
    assert abs((x ** 3).mean()) < 0.03 and abs((x ** 4).mean() - 3.0) < 0.1
    assert np.isfinite(x).all()


def test_workload_tables():
    w = I.WORKLOADS
    assert w["C1"].flops() == 4 * 64 * 2 * 128 * 128
    assert w["C3"].flops() == 4 * 128 * 4 * 32 * (4096 * 4097 // 2)
    assert w["C3"].dense_flops() == 2 * (w["C3"].flops() - 4 * 128 * 4 * 32 * 4096 / 2)
    assert abs(w["C2"].bytes() / 1e6 - 269.48) < 0.01
    assert abs(w["C3"].scale - 128 ** -0.5) < 1e-15


def test_make_qkv_c1_and_shifted_keys():
    w = I.WORKLOADS["C1"]
    q, k, v = I.make_qkv(w)
    assert q.shape == (1, 2, 128, 64) and k.shape == v.shape == (1, 2, 128, 64) and q.dtype == np.uint16
    q2, _, _ = I.make_qkv(w)
    np.testing.assert_array_equal(q, q2)
    small = I.Workload("t", 1, 4, 2, 256, 256, 64, False, 5, sigma=0.5, k_shift=True)
    qs, ks, vs = I.make_qkv(small)
    kf = I.bf16_bits_to_f32(ks)
    assert abs(I.bf16_bits_to_f32(vs).std() - 0.5) < 0.01
    means = kf.mean(axis=(0, 2, 3))
    c = I.normal_stream(5, 4 * 256 * 64 + 2 * 2 * 256 * 64, 2)
    np.testing.assert_allclose(means, c, atol=0.02)          # per-kv-head constant shift


def test_sample_rows():
    w = I.WORKLOADS["C3"]
    r = I.sample_rows(I.Workload("t", 1, 3, 1, 4096, 4096, 128, True, 9), 64)
    assert r.shape == (3, 64) and r.dtype == np.int32
    for row in r:
        assert len(set(row.tolist())) == 64 and (np.diff(row) > 0).all()
        assert {0, 1, 63, 64, 127, 128, 255, 256, 4094, 4095} <= set(row.tolist())
    assert not np.array_equal(r[0], r[1])
    tiny = I.sample_rows(I.Workload("t", 1, 1, 1, 5, 5, 64, True, 9), 64)
    assert tiny.tolist() == [[0, 1, 2, 3, 4]]
    assert w.check_rows == 0 and I.WORKLOADS["C2"].check_rows == 0        # every row of C2 and C3 is checked
    assert I.WORKLOADS["C4"].check_rows == 512 and I.WORKLOADS["C5"].check_rows == 256
