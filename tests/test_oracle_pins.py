"""Pins for the fp64 CPU reference (oracle/attn_ref.c).

Nothing here compares the reference with itself: every test checks it against
something the definition of attention (the paper's "Motivating Example": S = QK^T, P = softmax(S),
O = PV), the causal GQA workload (Evaluation, "Kernel Performance") or plain mathematics fixes -- hand
worked values, closed forms, invariants, brute force in pure Python, an
independent library routine on tiny inputs.  Each pin is chosen so that a
plausible slip (dropped scale, wrong head map, off-by-one mask, transposed
operand, LSE in the wrong base or of unscaled scores) fails at least one test.
"""
import math
import os

import numpy as np
import pytest

from oracle import attn_ref, attn_ref_row_probs
from paper_2604_18616_amd.inputs import bf16_bits_to_f32, f32_to_bf16_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rnd(shape, seed, sigma=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * sigma


def bits(x):
    return f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def widen(h):
    return bf16_bits_to_f32(h).astype(np.float64)


def brute_force(q, k, v, causal, scale):
    """Pure-Python loops, naive order, no max subtraction (tiny inputs only)."""
    B, Hq, Sq, D = q.shape
    _, Hkv, Sk, _ = k.shape
    g = Hq // Hkv
    o = np.zeros((B, Hq, Sq, D))
    lse = np.full((B, Hq, Sq), -math.inf)
    for b in range(B):
        for h in range(Hq):
            hk = h // g
            for i in range(Sq):
                js = [j for j in range(Sk) if (not causal) or j <= i + (Sk - Sq)]
                if not js:
                    continue
                e = []
                for j in js:
                    s = 0.0
                    for d in range(D):
                        s += float(q[b, h, i, d]) * float(k[b, hk, j, d])
                    e.append(math.exp(scale * s))
                tot = sum(e)
                lse[b, h, i] = math.log(tot)
                for d in range(D):
                    o[b, h, i, d] = sum(e[n] * float(v[b, hk, j, d]) for n, j in enumerate(js)) / tot
    return o, lse


# ---------------------------------------------------------------- worked values
def _read_kv(path):
    out = {}
    with open(path) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, val = line.split()
                out[name] = float(val)
    return out


def test_hand_example_d1():
    g = _read_kv(os.path.join(GOLDEN, "hand_example_d1.txt"))
    q = np.array(g["q"]).reshape(1, 1, 1, 1)
    k = np.array([g["k0"], g["k1"]]).reshape(1, 1, 2, 1)
    v = np.array([g["v0"], g["v1"]]).reshape(1, 1, 2, 1)
    o, lse = attn_ref(q, k, v, False, 1.0)
    assert o[0, 0, 0, 0] == pytest.approx(g["o"], abs=1e-14)
    assert lse[0, 0, 0] == pytest.approx(g["lse"], abs=1e-14)
    # the same example with scale = 2 and keys halved must give the same answer
    o2, lse2 = attn_ref(q, k / 2.0, v, False, 2.0)
    assert o2[0, 0, 0, 0] == pytest.approx(g["o"], abs=1e-14)
    assert lse2[0, 0, 0] == pytest.approx(g["lse"], abs=1e-14)


def test_hand_example_probs_bf16_path():
    # k1 = ln 2 is not a bf16 number; use q = 2, k = (0, 1): s = (0, 2) at scale 1
    q, k, v = bits([[[[2.0]]]]), bits([[[[0.0], [1.0]]]]), bits([[[[0.0], [3.0]]]])
    p, orow, lse = attn_ref_row_probs(q, k, v, False, 1.0, 0, 0, 0)
    e2 = math.exp(2.0)
    assert p[0] == pytest.approx(1.0 / (1.0 + e2), abs=1e-15)
    assert p[1] == pytest.approx(e2 / (1.0 + e2), abs=1e-15)
    assert orow[0] == pytest.approx(3.0 * e2 / (1.0 + e2), abs=1e-14)
    assert lse == pytest.approx(math.log(1.0 + e2), abs=1e-14)


def test_uniform_keys_closed_form_golden():
    rows = np.loadtxt(os.path.join(GOLDEN, "uniform_keys.txt"))
    S = rows.shape[0]
    q = np.zeros((1, 1, S, 4))
    k = rnd((1, 1, S, 4), 3)
    v = np.arange(S, dtype=np.float64).reshape(1, 1, S, 1)
    v = np.concatenate([v, -v, 2 * v, v * 0 + 7], axis=3)[:, :, :, :4]
    o, lse = attn_ref(q, k, v, True, 0.5)
    np.testing.assert_allclose(o[0, 0, :, 0], rows[:, 1], atol=1e-13)
    np.testing.assert_allclose(o[0, 0, :, 1], -rows[:, 1], atol=1e-13)
    np.testing.assert_allclose(o[0, 0, :, 3], 7.0, atol=1e-13)
    np.testing.assert_allclose(lse[0, 0], rows[:, 2], atol=1e-13)


# ---------------------------------------------------------------- invariants
@pytest.mark.parametrize("causal", [False, True])
def test_softmax_rows_sum_to_one(causal):
    q, k, v = bits(rnd((2, 4, 9, 16), 1)), bits(rnd((2, 2, 13, 16), 2)), bits(rnd((2, 2, 13, 16), 3))
    for (b, h, i) in [(0, 0, 0), (1, 3, 8), (0, 2, 4)]:
        p, orow, lse = attn_ref_row_probs(q, k, v, causal, 0.25, b, h, i)
        assert abs(p.sum() - 1.0) < 1e-14
        assert (p >= 0).all()
        nvis = 13 if not causal else i + (13 - 9) + 1
        assert (p[nvis:] == 0).all() and (p[:nvis] > 0).all()
        # O row must be the P-weighted sum of that kv head's V rows
        np.testing.assert_allclose(orow, p @ widen(v)[b, h // 2], atol=1e-14)
        # and p must equal exp(s - lse) for the scaled scores
        s = 0.25 * (widen(k)[b, h // 2] @ widen(q)[b, h, i])
        np.testing.assert_allclose(p[:nvis], np.exp(s[:nvis] - lse), rtol=1e-12)


@pytest.mark.parametrize("causal", [False, True])
def test_constant_v_gives_constant_output(causal):
    q, k = bits(rnd((1, 2, 17, 8), 4)), bits(rnd((1, 2, 17, 8), 5))
    v = bits(np.full((1, 2, 17, 8), 1.25))
    o, _ = attn_ref(q, k, v, causal, 0.3)
    assert np.abs(o - 1.25).max() < 1e-12


def test_causal_row0_is_v0():
    q, k, v = bits(rnd((2, 4, 12, 8), 6)), bits(rnd((2, 2, 12, 8), 7)), bits(rnd((2, 2, 12, 8), 8))
    o, lse = attn_ref(q, k, v, True, 0.35)
    vq = np.repeat(widen(v), 2, axis=1)
    np.testing.assert_allclose(o[:, :, 0, :], vq[:, :, 0, :], atol=1e-15)
    s00 = 0.35 * np.einsum("bhd,bhd->bh", widen(q)[:, :, 0, :], np.repeat(widen(k), 2, axis=1)[:, :, 0, :])
    np.testing.assert_allclose(lse[:, :, 0], s00, atol=1e-13)


def test_single_key():
    q, k, v = rnd((1, 3, 5, 4), 9), rnd((1, 3, 1, 4), 10), rnd((1, 3, 1, 4), 11)
    o, lse = attn_ref(q, k, v, False, 0.7)
    np.testing.assert_allclose(o, np.broadcast_to(v, o.shape), atol=1e-15)
    np.testing.assert_allclose(lse, 0.7 * np.einsum("bhid,bhd->bhi", q, k[:, :, 0, :]), atol=1e-13)


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(1, 1, 1, 3, 5, 2), (2, 4, 2, 6, 6, 3), (1, 6, 2, 4, 7, 5), (1, 2, 1, 7, 4, 2)])
def test_against_pure_python_brute_force(shape, causal):
    B, Hq, Hkv, Sq, Sk, D = shape
    q, k, v = rnd((B, Hq, Sq, D), 20, 0.7), rnd((B, Hkv, Sk, D), 21, 0.7), rnd((B, Hkv, Sk, D), 22)
    o, lse = attn_ref(q, k, v, causal, 0.9)
    ob, lb = brute_force(q, k, v, causal, 0.9)
    np.testing.assert_allclose(o, ob, atol=1e-13)
    fin = np.isfinite(lb)
    np.testing.assert_allclose(lse[fin], lb[fin], atol=1e-13)
    assert (lse[~fin] == -np.inf).all()                      # rows with no visible key
    if causal and Sq > Sk:
        assert (~fin).any() and (o[~fin] == 0).all()


def test_bf16_entry_equals_f64_entry_on_widened_bits():
    # the bf16 entry point must widen exactly and then follow the same definition
    qb, kb, vb = bits(rnd((1, 4, 10, 8), 30)), bits(rnd((1, 2, 11, 8), 31)), bits(rnd((1, 2, 11, 8), 32))
    o1, l1 = attn_ref(qb, kb, vb, True, 0.4)
    ob, lb = brute_force(widen(qb), widen(kb), widen(vb), True, 0.4)
    np.testing.assert_allclose(o1, ob, atol=1e-13)
    np.testing.assert_allclose(l1, lb, atol=1e-13)


def test_library_second_opinion_torch_fp64():
    torch = pytest.importorskip("torch")
    q, k, v = rnd((2, 3, 33, 16), 40), rnd((2, 3, 47, 16), 41), rnd((2, 3, 47, 16), 42)
    o, lse = attn_ref(q, k, v, False, 0.25)
    tq, tk, tv = (torch.from_numpy(x) for x in (q, k, v))
    s = 0.25 * tq @ tk.transpose(-1, -2)
    np.testing.assert_allclose(o, (torch.softmax(s, -1) @ tv).numpy(), atol=1e-12)
    np.testing.assert_allclose(lse, torch.logsumexp(s, -1).numpy(), atol=1e-12)


# ---------------------------------------------------------------- metamorphic
def test_score_shift_moves_lse_only():
    # adding c to every component of every key shifts score (i,j) by scale*c*sum_d q_id for all j
    q, k, v = rnd((1, 2, 9, 8), 50), rnd((1, 2, 12, 8), 51), rnd((1, 2, 12, 8), 52)
    c, scale = 3.5, 0.6
    o0, l0 = attn_ref(q, k, v, False, scale)
    o1, l1 = attn_ref(q, k + c, v, False, scale)
    np.testing.assert_allclose(o1, o0, atol=1e-11)
    np.testing.assert_allclose(l1 - l0, scale * c * q.sum(-1), atol=1e-11)


def test_large_scores_do_not_overflow():
    # scores of +-700 overflow exp() unless the maximum is subtracted first
    q = np.full((1, 1, 2, 1), 1.0)
    k = np.array([700.0, 699.0, -700.0]).reshape(1, 1, 3, 1)
    v = np.array([1.0, 2.0, 5.0]).reshape(1, 1, 3, 1)
    o, lse = attn_ref(q, k, v, False, 1.0)
    e = math.exp(-1.0)
    assert o[0, 0, 0, 0] == pytest.approx((1.0 + 2.0 * e) / (1.0 + e), abs=1e-13)
    assert lse[0, 0, 0] == pytest.approx(700.0 + math.log1p(e), abs=1e-11)


def test_key_permutation_invariance_noncausal():
    q, k, v = rnd((1, 2, 7, 8), 60), rnd((1, 1, 19, 8), 61), rnd((1, 1, 19, 8), 62)
    perm = np.random.default_rng(63).permutation(19)
    o0, l0 = attn_ref(q, k, v, False, 0.5)
    o1, l1 = attn_ref(q, k[:, :, perm], v[:, :, perm], False, 0.5)
    np.testing.assert_allclose(o1, o0, atol=1e-13)
    np.testing.assert_allclose(l1, l0, atol=1e-13)


def test_gqa_equals_mha_with_repeated_kv_heads():
    q, k, v = rnd((2, 6, 8, 4), 70), rnd((2, 2, 8, 4), 71), rnd((2, 2, 8, 4), 72)
    o0, l0 = attn_ref(q, k, v, True, 0.5)
    # contiguous groups: q heads 0..2 -> kv head 0, 3..5 -> kv head 1
    o1, l1 = attn_ref(q, np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1), True, 0.5)
    np.testing.assert_array_equal(o0, o1)
    np.testing.assert_array_equal(l0, l1)
    # an interleaved map (h % Hkv) is a different function: make sure we would notice
    o2, _ = attn_ref(q, np.tile(k, (1, 3, 1, 1)), np.tile(v, (1, 3, 1, 1)), True, 0.5)
    assert np.abs(o2 - o0).max() > 1e-3


@pytest.mark.parametrize("Sq,Sk", [(8, 8), (5, 11), (11, 5)])
def test_causal_equals_dense_softmax_with_explicit_mask(Sq, Sk):
    q, k, v = rnd((1, 2, Sq, 4), 80), rnd((1, 2, Sk, 4), 81), rnd((1, 2, Sk, 4), 82)
    o, lse = attn_ref(q, k, v, True, 0.5)
    s = 0.5 * np.einsum("bhid,bhjd->bhij", q, k)
    i, j = np.arange(Sq)[:, None], np.arange(Sk)[None, :]
    vis = j <= i + (Sk - Sq)                          # bottom-right aligned
    e = np.where(vis, np.exp(s), 0.0)
    tot = e.sum(-1)
    ok = tot > 0
    oo = np.einsum("bhij,bhjd->bhid", e, v)
    np.testing.assert_allclose(o[ok], oo[ok] / tot[ok][:, None], atol=1e-13)
    np.testing.assert_allclose(lse[ok], np.log(tot[ok]), atol=1e-13)
    assert (o[~ok] == 0).all() and (lse[~ok] == -np.inf).all()
    if Sq == Sk:                                      # ordinary lower-triangular mask
        assert (vis == np.tril(np.ones((Sq, Sk), bool))).all()


def test_split_kv_merge_by_lse():
    # attention over [K1;K2] = LSE-weighted merge of the halves: pins LSE's base and scaling
    q, k, v = rnd((1, 2, 6, 8), 90), rnd((1, 2, 14, 8), 91), rnd((1, 2, 14, 8), 92)
    o, lse = attn_ref(q, k, v, False, 0.45)
    o1, l1 = attn_ref(q, k[:, :, :5], v[:, :, :5], False, 0.45)
    o2, l2 = attn_ref(q, k[:, :, 5:], v[:, :, 5:], False, 0.45)
    lm = np.logaddexp(l1, l2)
    om = np.exp(l1 - lm)[..., None] * o1 + np.exp(l2 - lm)[..., None] * o2
    np.testing.assert_allclose(lse, lm, atol=1e-13)
    np.testing.assert_allclose(o, om, atol=1e-13)


def test_large_scale_selects_argmax_key():
    q, k, v = rnd((1, 1, 5, 8), 100), rnd((1, 1, 9, 8), 101), rnd((1, 1, 9, 8), 102)
    o, _ = attn_ref(q, k, v, False, 1e4)
    jstar = np.einsum("id,jd->ij", q[0, 0], k[0, 0]).argmax(-1)
    np.testing.assert_allclose(o[0, 0], v[0, 0, jstar], atol=1e-9)


def test_row_subset_matches_full_rows_semantics():
    # rows=... must select query rows per (b,h) -- checked against brute force, not against rows=None
    q, k, v = rnd((1, 2, 9, 4), 110), rnd((1, 1, 9, 4), 111), rnd((1, 1, 9, 4), 112)
    rows = np.array([[0, 4, 8], [1, 2, 7]], dtype=np.int32)
    o, lse = attn_ref(q, k, v, True, 0.5, rows=rows)
    ob, lb = brute_force(q, k, v, True, 0.5)
    for h in range(2):
        np.testing.assert_allclose(o[0, h], ob[0, h, rows[h]], atol=1e-13)
        np.testing.assert_allclose(lse[0, h], lb[0, h, rows[h]], atol=1e-13)


def test_bad_arguments_raise():
    q, k, v = rnd((1, 3, 4, 4), 1), rnd((1, 2, 4, 4), 2), rnd((1, 2, 4, 4), 3)
    with pytest.raises(RuntimeError):
        attn_ref(q, k, v, False, 1.0)                  # Hq % Hkv != 0
    with pytest.raises(RuntimeError):
        attn_ref(rnd((1, 2, 4, 4), 1), k, v, False, 1.0, rows=[4])   # row out of range
