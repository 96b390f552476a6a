"""Parity of the HIP attention forward (through the C ABI) with the fp64 CPU reference.

Same seeded inputs on both sides, element-by-element comparison at the stated bar:
max-abs <= 2e-2 and mean-abs <= 2e-3 on O, max-abs <= 1e-3 on LSE.
"""
import numpy as np
import pytest

from paper_2604_18616_amd import inputs as I
from tests._util import check, oracle_parallel, run_hip

pytestmark = pytest.mark.gpu


def small(name, B, Hq, Hkv, Sq, Sk, D, causal, seed, **kw):
    return I.Workload(name, B, Hq, Hkv, Sq, Sk, D, causal, seed, **kw)


SMALL_CASES = [
    # several 128-row query tiles and 64-key tiles, ragged tails on both axes
    small("ragged_d128", 2, 4, 2, 200, 333, 128, False, 11),
    small("ragged_d128_causal", 2, 4, 2, 200, 333, 128, True, 12),
    small("ragged_d64", 1, 6, 2, 257, 321, 64, False, 13),
    small("ragged_d64_causal", 1, 6, 2, 257, 321, 64, True, 14),
    small("square_causal_d128", 1, 8, 2, 512, 512, 128, True, 15),
    small("square_causal_d64", 2, 2, 2, 384, 384, 64, True, 16),
    # degenerate sizes
    small("one_query", 2, 4, 4, 1, 500, 128, False, 17),
    small("one_query_causal", 2, 4, 1, 1, 500, 64, True, 18),
    small("one_key", 1, 2, 2, 130, 1, 128, False, 19),
    small("one_by_one", 1, 1, 1, 1, 1, 64, True, 20),
    small("more_queries_than_keys_causal", 1, 2, 1, 300, 100, 128, True, 21),   # rows 0..199 see no key
    small("exact_tiles", 1, 2, 2, 128, 64, 64, False, 22),
    # shifted keys stress the max subtraction (large common offset in every score of a row)
    small("shifted_keys", 1, 4, 4, 256, 640, 64, False, 23, sigma=0.5, k_shift=True),
    small("gqa8", 1, 8, 1, 256, 256, 128, True, 24),
    # ragged key counts through the 256-row kernel (Sq > 64): partial last tile, fewer keys than a tile
    small("ragged_keys_lt_tile", 1, 4, 2, 300, 37, 128, False, 25),
    small("ragged_keys_tile_plus_one", 2, 2, 1, 130, 65, 64, False, 26),
    small("ragged_keys_causal_long", 1, 4, 1, 700, 1000, 128, True, 27),
    small("ragged_keys_causal_d64", 1, 4, 2, 513, 449, 64, True, 28),
    small("ragged_both_noncausal", 2, 3, 3, 1001, 1003, 128, False, 29),
    small("queries_65", 1, 2, 2, 65, 320, 128, True, 30),
    # one kv head whose workgroups span several XCDs: the causal tile order alternates long and short tiles (5 and 6 tiles)
    small("mqa16_causal_5_tiles", 1, 16, 1, 1280, 1280, 128, True, 31),
    small("mqa16_causal_6_tiles_d64", 1, 16, 1, 1500, 1500, 64, True, 32),
]


def test_config_c1_full():
    w = I.WORKLOADS["C1"]
    q, k, v = I.make_qkv(w)
    o, lse = run_hip(q, k, v, w.causal, w.scale)
    o_ref, lse_ref = oracle_parallel(q, k, v, w.causal, w.scale)
    print(w.name, check(o, lse, o_ref, lse_ref, w.name))


@pytest.mark.parametrize("wg_rows", [0, 128, 256])
@pytest.mark.parametrize("w", SMALL_CASES, ids=lambda w: w.name)
def test_small_shapes_full_oracle(w, wg_rows):
    """Every small shape through attn_fwd (the library picks the workgroup shape) and through attn_fwd_tile with
    the 128-row (4 wavefronts, several workgroups per CU) and the 256-row (8 wavefronts) workgroup forced."""
    q, k, v = I.make_qkv(w)
    o, lse = run_hip(q, k, v, w.causal, w.scale, wg_rows=wg_rows)
    o_ref, lse_ref = oracle_parallel(q, k, v, w.causal, w.scale)
    print(w.name, wg_rows, check(o, lse, o_ref, lse_ref, w.name))
    if w.causal and w.Sq > w.Sk:
        assert (lse[:, :, : w.Sq - w.Sk] == -np.inf).all() and (o[:, :, : w.Sq - w.Sk] == 0).all()


def test_scale_other_than_rsqrt_d_and_null_lse():
    w = small("scale", 1, 2, 1, 192, 192, 128, True, 31)
    q, k, v = I.make_qkv(w)
    o, lse = run_hip(q, k, v, True, 0.2)
    o_ref, lse_ref = oracle_parallel(q, k, v, True, 0.2)
    check(o, lse, o_ref, lse_ref, "scale=0.2")
    o2, lse2 = run_hip(q, k, v, True, 0.2, want_lse=False)
    assert np.array_equal(o2, o) and np.isnan(lse2).all()      # lse untouched when NULL is passed


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("D,Sq,Sk", [(128, 300, 300), (64, 200, 333), (128, 40, 130)])
def test_strided_layout_of_the_papers_kernel(D, Sq, Sk, causal):
    """attn_fwd_strided on [B, S, H, D] buffers (the [seq, head, d] layout of the paper's
    Figure 1 with a batch dimension), output written in the same layout, plus a padded row
    stride; compared with the reference on the equivalent [B, H, S, D] arrays."""
    import torch
    from paper_2604_18616_amd import binding
    B, Hq, Hkv = 2, 4, 2
    w = small("strided", B, Hq, Hkv, Sq, Sk, D, causal, 41)
    qb, kb, vb = I.make_qkv(w)                                   # [B,H,S,D]
    dev = lambda a: torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    q_bshd = dev(np.ascontiguousarray(qb.transpose(0, 2, 1, 3)))  # [B,S,H,D] storage
    k_bshd = dev(np.ascontiguousarray(kb.transpose(0, 2, 1, 3)))
    pad = torch.full((B, Hkv, Sk, D + 16), float("nan"), dtype=torch.bfloat16, device="cuda")   # padded rows for V
    pad[..., :D] = dev(vb)
    o_bshd = torch.full((B, Sq, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda")
    binding.attn_fwd(q_bshd.transpose(1, 2), k_bshd.transpose(1, 2), pad[..., :D], o_bshd.transpose(1, 2), lse,
                     causal=causal, scale=w.scale)
    torch.cuda.synchronize()
    o = I.bf16_bits_to_f32(o_bshd.transpose(1, 2).contiguous().view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
    o_ref, lse_ref = oracle_parallel(qb, kb, vb, causal, w.scale)
    print(check(o, lse.cpu().numpy().astype(np.float64), o_ref, lse_ref, "strided"))
    assert torch.isnan(pad[..., D:].float()).all()              # padding untouched


@pytest.mark.parametrize("wg_rows", [128, 256])
@pytest.mark.parametrize("direction", ["rising", "falling", "spike"])
@pytest.mark.parametrize("causal", [False, True])
def test_scores_far_from_the_first_tile_maximum(direction, causal, wg_rows):
    """The kernel exponentiates against a stale reference and only re-bases when a partial sum
    would overflow: drive the scores hundreds of binades away from the first tile's maximum
    (upwards: forces re-basing several times; downwards: everything after the first tiles
    underflows against the reference; spike: one huge score in the middle of a late tile)."""
    B, Hq, Hkv, S, D = 1, 2, 1, 1024, 128
    rng = np.random.default_rng(77)
    q = rng.standard_normal((B, Hq, S, D)).astype(np.float32)
    k = rng.standard_normal((B, Hkv, S, D)).astype(np.float32)
    v = rng.standard_normal((B, Hkv, S, D)).astype(np.float32)
    u = np.ones(D, dtype=np.float32) / np.sqrt(D)
    q = q + 40.0 * u                                 # every query has a large component along u
    ramp = np.linspace(0.0, 1.0, S, dtype=np.float32)[None, None, :, None]
    if direction == "rising":
        k = k + 60.0 * ramp * u                      # q.k grows by ~2400 -> ~300 binades after scaling
    elif direction == "falling":
        k = k + 60.0 * (1.0 - ramp) * u
    else:
        k[:, :, 777, :] += 80.0 * u
    qb, kb, vb = (I.f32_to_bf16_bits(x) for x in (q, k, v))
    scale = D ** -0.5
    o, lse = run_hip(qb, kb, vb, causal, scale, wg_rows=wg_rows)
    o_ref, lse_ref = oracle_parallel(qb, kb, vb, causal, scale)
    print(direction, causal, wg_rows, check(o, lse, o_ref, lse_ref, direction))


def whole_tensor_properties(w, o, lse, v):
    """Properties that hold for every row at any size: finite outputs, O inside the hull of V, causal row 0 = V[0]."""
    assert np.isfinite(o).all() and np.isfinite(lse).all()
    vf = I.bf16_bits_to_f32(v).astype(np.float64)
    g = w.Hq // w.Hkv
    if w.causal and w.Sq == w.Sk:                  # first query row attends to key 0 only
        assert np.array_equal(o[:, :, 0, :], np.repeat(vf[:, :, 0, :], g, axis=1))
    vmax = np.repeat(np.abs(vf).max(axis=2), g, axis=1)[:, :, None, :]
    assert (np.abs(o) <= vmax * (1 + 2 ** -7)).all()   # O is a convex combination of V rows


@pytest.mark.parametrize("name", ["C2", "C3"])
def test_full_size_configs_every_row(name):
    """C2 and the headline C3 at full size, in the launch configuration the bench times: EVERY query row of every
    head against the reference (the benchmark definition states sampling only for C4 and C5)."""
    w = I.WORKLOADS[name]
    assert w.check_rows == 0
    q, k, v = I.make_qkv(w)
    o, lse = run_hip(q, k, v, w.causal, w.scale)
    o_ref, lse_ref = oracle_parallel(q, k, v, w.causal, w.scale)
    print(name, check(o, lse, o_ref, lse_ref, name), "rows checked:", w.B * w.Hq * w.Sq)
    whole_tensor_properties(w, o, lse, v)


@pytest.mark.parametrize("name,wg_rows", [("C4", 0), ("C5", 0), ("P1024", 0), ("P4096", 0), ("P16384", 0), ("N8K", 0),
                                          ("C4", 256), ("C5", 128), ("P1024", 128)])
def test_full_size_configs_sampled_rows(name, wg_rows):
    """C4 (512 rows per head) and C5 (256), as the benchmark definition states, and the shapes of the paper's own
    attention workload (Evaluation, "Kernel Performance"; x-axis of Figure 3a: batch 16, 8 query heads on 1 kv
    head, d = 128, causal, sequence 1024 / 4096 / 16384) plus the long non-causal case, 64 rows per head: the
    reference on seeded sample rows (always including tile edges and the causal extremes) and the whole-tensor
    properties on every row."""
    w = I.WORKLOADS[name]
    q, k, v = I.make_qkv(w)
    rows = I.sample_rows(w, w.check_rows)
    o, lse = run_hip(q, k, v, w.causal, w.scale, wg_rows=wg_rows)   # 0: the shape the bench times; else the other one
    o_ref, lse_ref = oracle_parallel(q, k, v, w.causal, w.scale, rows=rows)
    idx = rows.reshape(w.B, w.Hq, -1)
    o_s = np.take_along_axis(o, idx[..., None], axis=2)
    lse_s = np.take_along_axis(lse, idx, axis=2)
    print(name, check(o_s, lse_s, o_ref, lse_ref, name), "rows per head:", idx.shape[-1])
    whole_tensor_properties(w, o, lse, v)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("D,Sq,Sk", [(128, 300, 70), (64, 333, 150), (128, 200, 333)])
def test_heads_of_4_gib_or_more_take_the_128_row_kernel_with_several_query_tiles(D, Sq, Sk, causal):
    """attn_fwd_strided with a V row pitch so large that one head of V spans 4 GiB or more: tile offsets no longer
    fit the 32-bit scalars of the 256-row kernel, and the launcher takes the 128-row kernel with 64-bit addressing
    for ANY query count -- here three query tiles, heads interleaved inside the rows ([seq, head, d] storage).
    The V buffer is a few GiB of untouched device memory with Sk * Hkv * D live elements."""
    import torch
    from paper_2604_18616_amd import binding
    B, Hq, Hkv = 1, 4, 2
    w = small("huge_pitch", B, Hq, Hkv, Sq, Sk, D, causal, 51)
    qb, kb, vb = I.make_qkv(w)
    pitch = -(-(1 << 32) // (2 * (Sk + 64))) + 8
    pitch += -pitch % 8                                          # elements; (Sk + 64) * pitch * 2 >= 2^32
    assert (Sk + 64) * pitch * 2 >= 1 << 32 and pitch < 1 << 28
    print("huge pitch", D, Sq, Sk, causal, "V pitch", pitch, "elements,", Sk * pitch * 2 >> 20, "MiB", flush=True)
    dev = lambda a: torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    q, k = dev(qb), dev(kb)
    vbuf = torch.empty((Sk - 1) * pitch + Hkv * D, dtype=torch.bfloat16, device="cuda")
    v = vbuf.as_strided((B, Hkv, Sk, D), (0, D, pitch, 1))      # row j of head h at j * pitch + h * D
    v.copy_(dev(vb))
    o = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full(q.shape[:3], float("nan"), dtype=torch.float32, device="cuda")
    binding.attn_fwd(q, k, v, o, lse, causal=causal, scale=w.scale)
    torch.cuda.synchronize()
    del vbuf, v
    o_h = I.bf16_bits_to_f32(o.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
    o_ref, lse_ref = oracle_parallel(qb, kb, vb, causal, w.scale)
    print(check(o_h, lse.cpu().numpy().astype(np.float64), o_ref, lse_ref, "huge_pitch"))
    if causal and Sq > Sk:
        assert (lse[:, :, : Sq - Sk] == -np.inf).all() and (o[:, :, : Sq - Sk] == 0).all()


def test_mfma_calibration_kernels_run_and_count_their_flops():
    """The measurement aids of the bench: every operand kind launches, finishes and reports the FLOPs it issued
    (8 or 4 wavefronts per workgroup x 4 or 8 MFMAs of 32768 flop per iteration, or as many FLOPs in 16x16x32)."""
    import torch

    from paper_2604_18616_amd import binding
    lib = binding.load_library()
    sink = torch.zeros(16, dtype=torch.float32, device="cuda:0")
    sp = torch.cuda.current_stream().cuda_stream
    assert lib.attn_mfma_calibration(sink.data_ptr(), 64, 100, sp) == 64 * 8 * 100 * 4 * 32768.0
    for data, waves, per_iter in ((0, 8, 4), (1, 8, 8), (2, 8, 8), (3, 8, 8), (4, 4, 8), (5, 4, 8)):
        print("calibration kind", data, flush=True)
        assert lib.attn_mfma_calibration_data(sink.data_ptr(), 64, 100, data, sp) == 64 * waves * 100 * per_iter * 32768.0
    torch.cuda.synchronize()
    assert float(sink.abs().sum()) == 0.0            # the sink is never written in practice


@pytest.mark.parametrize("kind", ["zeros", "constants"])
@pytest.mark.parametrize("causal", [False, True])
def test_uniform_scores(kind, causal):
    """Degenerate inputs: every score of a row is equal (all-zero tensors, or one constant per tensor), so the softmax
    is uniform over the visible keys, O is the mean of V (the constant) and LSE = score + log(number of visible keys).
    Checked against the reference and against that closed form; ragged sizes through the 256-row kernel."""
    w = small("uniform_" + kind, 1, 4, 2, 300, 333, 128, causal, 41)
    q, k, v = I.make_qkv(w)
    cq, ck, cv = (0.0, 0.0, 0.0) if kind == "zeros" else (0.5, 0.25, 1.5)
    for arr, c in ((q, cq), (k, ck), (v, cv)):
        arr[...] = I.f32_to_bf16_bits(np.full(1, c, dtype=np.float32))[0]
    o, lse = run_hip(q, k, v, w.causal, w.scale)
    o_ref, lse_ref = oracle_parallel(q, k, v, w.causal, w.scale)
    print(w.name, check(o, lse, o_ref, lse_ref, w.name))
    visible = np.clip(np.arange(w.Sq) + (w.Sk - w.Sq) + 1, 0, w.Sk) if causal else np.full(w.Sq, w.Sk)
    assert visible.min() >= 1
    assert np.abs(o - cv).max() <= 2.0 ** -8 * abs(cv)                       # the mean of a constant, rounded once to bf16
    want = cq * ck * w.D * w.scale + np.log(visible)
    assert np.abs(lse - want[None, None, :]).max() <= 1e-3
