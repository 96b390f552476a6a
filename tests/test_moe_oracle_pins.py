"""Pins of the MoE reference (oracle/moe_ref.c) to things other than itself: the e4m3 format's
published code values, brute-force nearest-code checks of the encoder, tie and clamp cases, the
quantization recipe's invariants, an independent dequantize-then-matmul formulation in numpy,
and structural invariants (routing, slot order, linearity, zero gates)."""
import math
import os

import numpy as np
import pytest

import oracle
from paper_2604_18616_amd import inputs as I

GOLD = os.path.join(os.path.dirname(__file__), "golden", "e4m3_codes.txt")
VALS = np.array([oracle.e4m3_decode(c) for c in range(256)])


def small(T=12, seed=3, **kw):
    cfg = dict(H=256, I=128, E=4, KTOP=2, EP=2)
    cfg.update(kw)
    w = I.MoeWorkload("t", T, seed, **cfg)
    return w, I.make_moe(w)


def test_decode_matches_the_published_format():
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        code, val = line.split()
        got = oracle.e4m3_decode(int(code, 16))
        assert got == float(val) and math.copysign(1, got) == math.copysign(1, float(val)), (code, got)
    assert math.isnan(oracle.e4m3_decode(0x7F)) and math.isnan(oracle.e4m3_decode(0xFF))
    pos = VALS[:127]
    assert np.all(np.diff(pos) > 0) and np.array_equal(VALS[128:255], -pos)     # ordered, symmetric
    assert np.array_equal(I.e4m3_values()[:127], pos)                              # the input generator's table agrees


def test_encode_round_trips_every_finite_code():
    for c in list(range(0, 127)) + list(range(128, 255)):
        assert oracle.e4m3_encode(VALS[c]) == c, c


def test_encode_is_nearest_with_ties_to_even_and_clamps():
    rng = np.random.default_rng(1)
    vals = np.concatenate([rng.normal(0, 1, 500), rng.normal(0, 100, 500), rng.uniform(-0.05, 0.05, 500)]).astype(np.float32)
    finite = np.concatenate([VALS[:127], VALS[128:255]])
    for v in vals:
        got = oracle.e4m3_decode(oracle.e4m3_encode(v))
        best = np.abs(finite - np.clip(float(v), -448, 448)).min()
        assert abs(got - np.clip(float(v), -448, 448)) == best, v
    # exact midpoints go to the code with an even mantissa
    assert oracle.e4m3_encode(1.0625) == 0x38 and oracle.e4m3_encode(1.1875) == 0x3A
    assert oracle.e4m3_encode(-1.0625) == 0xB8
    assert oracle.e4m3_encode(2.0 ** -10) == 0x00 and oracle.e4m3_encode(3 * 2.0 ** -10) == 0x02
    assert oracle.e4m3_encode(15 * 2.0 ** -10) == 0x08                    # subnormal/normal boundary tie -> 2^-6
    assert oracle.e4m3_encode(464.0) == 0x7E and oracle.e4m3_encode(1e9) == 0x7E and oracle.e4m3_encode(-1e9) == 0xFE
    sweep = np.linspace(-500, 500, 20001).astype(np.float32)
    dec = np.array([oracle.e4m3_decode(oracle.e4m3_encode(v)) for v in sweep])
    assert np.all(np.diff(dec) >= 0)                                       # monotone


def test_group_quantization_recipe():
    rng = np.random.default_rng(2)
    v = rng.normal(0, 3, 128).astype(np.float32)
    code, scale = oracle.quant_group(v)
    amax = np.abs(v).max()
    assert scale == np.float32(amax) * np.float32(1.0 / 448.0)             # one fp32 multiplication
    assert VALS[code[np.abs(v).argmax()]] in (448.0, -448.0)                # the largest element uses the full range
    deq = VALS[code] * scale
    spacing = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(np.abs(deq / scale), 2.0 ** -6))) - 3), 2.0 ** -9)
    assert np.all(np.abs(deq - v) <= 0.5 * spacing * scale * (1 + 1e-6) + 1e-12)
    code0, scale0 = oracle.quant_group(np.zeros(128, dtype=np.float32))
    assert scale0 == 1.0 and not code0.any()
    code2, scale2 = oracle.quant_group(4 * v)                              # powers of two move into the scale
    assert np.array_equal(code2, code) and scale2 == 4 * scale


def numpy_moe(d, H, I_, E):
    """Independent formulation: dequantize weights and activations fully, then plain matmuls."""
    T, K = d["ids"].shape
    xf = I.bf16_bits_to_f32(d["x"])
    w13 = VALS[d["w13"]] * np.repeat(np.repeat(d["s13"].astype(np.float64), 128, axis=1), 128, axis=2)
    w2 = VALS[d["w2"]] * np.repeat(np.repeat(d["s2"].astype(np.float64), 128, axis=1), 128, axis=2)
    y = np.zeros((T, H))

    def deq(v):
        out = np.empty(v.shape[0])
        for b in range(v.shape[0] // 128):
            code, s = oracle.quant_group(v[128 * b:128 * b + 128])
            out[128 * b:128 * b + 128] = VALS[code] * float(s)
        return out

    for t in range(T):
        xd = deq(xf[t])
        for k in range(K):
            e = d["ids"][t, k]
            if e < 0 or e >= E:
                continue
            gu = w13[e] @ xd
            g, u = gu[:I_], gu[I_:]
            a = (g / (1 + np.exp(-g)) * u).astype(np.float32)
            y[t] += float(d["wts"][t, k]) * (w2[e] @ deq(a))
    return y


@pytest.mark.parametrize("cfg", [dict(), dict(H=384, I=256, E=3, KTOP=3, EP=1), dict(H=128, I=128, E=2, KTOP=1, EP=1)])
def test_against_dequantize_then_matmul(cfg):
    w, d = small(T=10, seed=11, **cfg)
    y = oracle.moe_ref(**d)
    want = numpy_moe(d, w.H, w.I, w.E)
    assert np.abs(want).max() > 0.05
    np.testing.assert_allclose(y, want, rtol=1e-9, atol=1e-12)


def test_tokens_without_a_local_expert_are_zero_and_rows_select():
    w, d = small(T=40, seed=5, EP=4)
    y = oracle.moe_ref(**d)
    remote = ~(d["ids"] >= 0).any(axis=1)
    assert remote.any() and (~remote).any()
    assert not y[remote].any() and np.all(np.abs(y[~remote]).max(axis=1) > 0)
    rows = np.array([3, 0, 39, 17], dtype=np.int32)
    assert np.array_equal(oracle.moe_ref(rows=rows, **d), y[rows])
    big = dict(d); big["ids"] = np.where(d["ids"] >= 0, d["ids"], w.E + 5)      # ids past the local range are remote too
    assert np.array_equal(oracle.moe_ref(**big), y)


def test_linear_in_the_routing_weights_and_down_scales():
    w, d = small(T=8, seed=6, EP=1)
    y = oracle.moe_ref(**d)
    d2 = dict(d); d2["s2"] = d["s2"] * np.float32(2)
    assert np.array_equal(oracle.moe_ref(**d2), 2 * y)
    d3 = dict(d); d3["wts"] = d["wts"] * np.float32(0.5)
    assert np.array_equal(oracle.moe_ref(**d3), 0.5 * y)
    one = dict(d); one["wts"] = d["wts"].copy(); one["wts"][:, 1] = 0
    two = dict(d); two["wts"] = d["wts"].copy(); two["wts"][:, 0] = 0
    np.testing.assert_allclose(oracle.moe_ref(**one) + oracle.moe_ref(**two), y, rtol=1e-12, atol=1e-15)


def test_slot_order_does_not_matter_and_zero_gates_give_zero():
    w, d = small(T=8, seed=7, EP=1)
    y = oracle.moe_ref(**d)
    sw = dict(d); sw["ids"] = d["ids"][:, ::-1].copy(); sw["wts"] = d["wts"][:, ::-1].copy()
    np.testing.assert_allclose(oracle.moe_ref(**sw), y, rtol=1e-12, atol=1e-15)
    z = dict(d); z["w13"] = d["w13"].copy(); z["w13"][:, :w.I, :] = 0           # gate rows come first: silu(0) * u = 0
    assert not oracle.moe_ref(**z).any()
    zu = dict(d); zu["w13"] = d["w13"].copy(); zu["w13"][:, w.I:, :] = 0         # up rows second
    assert not oracle.moe_ref(**zu).any()
    assert oracle.moe_ref(**d).any()


def test_staged_entry_points_compose_to_the_whole():
    """intermediate -> fp32 -> quant128 -> down -> weighted sum reproduces moe_ref; the intermediate also
    matches the dequantize-then-matmul formulation."""
    w, d = small(T=6, seed=12, EP=1, H=256, I=256)
    y = oracle.moe_ref(**d)
    t = 4
    want = np.zeros(w.H)
    for k in range(w.KTOP):
        e = int(d["ids"][t, k])
        a = oracle.moe_intermediate(d["x"], d["w13"], d["s13"], t, e)
        codes, scales = zip(*[oracle.quant_group(a[128 * b:128 * b + 128].astype(np.float32)) for b in range(w.I // 128)])
        want += float(d["wts"][t, k]) * oracle.moe_down(np.concatenate(codes), np.array(scales, dtype=np.float32), d["w2"], d["s2"], e)
    np.testing.assert_allclose(want, y[t], rtol=1e-13, atol=1e-15)
    # the intermediate against plain dequantized matmuls
    xf = I.bf16_bits_to_f32(d["x"][t])
    xd = np.concatenate([VALS[c] * s for c, s in (oracle.quant_group(xf[128 * b:128 * b + 128]) for b in range(w.H // 128))])
    e = int(d["ids"][t, 0])
    w13 = VALS[d["w13"][e]] * np.repeat(np.repeat(d["s13"][e].astype(np.float64), 128, axis=0), 128, axis=1)
    gu = w13 @ xd
    np.testing.assert_allclose(oracle.moe_intermediate(d["x"], d["w13"], d["s13"], t, e),
                               gu[:w.I] / (1 + np.exp(-gu[:w.I])) * gu[w.I:], rtol=1e-10, atol=1e-13)


def test_workload_table_and_generator():
    w = I.MOE_WORKLOADS["M1024"]
    assert (w.T, w.H, w.I, w.E, w.KTOP, w.EP) == (1024, 7168, 2048, 32, 4, 8)
    ws, d = small(T=64, seed=8, EP=8, E=4, KTOP=4)
    ids = d["ids"]
    assert ids.shape == (64, 4) and ids.max() < 4 and ids.min() == -1
    for row in ids:                                                             # distinct experts per token
        loc = row[row >= 0]
        assert len(set(loc.tolist())) == len(loc)
    np.testing.assert_allclose(d["wts"].sum(axis=1), 1.0, rtol=1e-6)
    v = VALS[d["w13"].ravel()]
    assert not np.isnan(v).any() and abs(v.mean()) < 2 and 55 < v.std() < 70    # ~ 64 N(0,1)
    assert ws.flops(ids) == 6.0 * 256 * 128 * (ids >= 0).sum()
