"""GPU parity of moe_ffn_fp8 (through the C ABI) against the fp64 reference, stage by stage.

Two things make an end-to-end tolerance meaningless here, so the path is checked in stages.

(a) The path contains two quantization decisions.  The first (input activations) is taken by
    both sides with the same fp32 recipe on the same bits: codes and scales must agree bit for
    bit.  The second (the gated intermediate) is taken on values the kernel accumulates on the
    matrix cores and the reference in fp64: where the two differ slightly a code may
    legitimately land on the neighbouring e4m3 value, an O(2^-4) change of that element.  As
    for any result that is not unique, what is unique is compared exactly and the rest is
    checked for validity.
(b) The FP8 matrix cores do not add exactly: measured on the device (random e4m3 operands,
    K = 64), one MFMA returns its 64-term sum with an error of up to 2^-11.2 times the LARGEST
    |product| of the sum (products are aligned to the largest one and cut; both FP8 MFMA forms
    give identical results).  This is the arithmetic of the method's "FP8 matrix cores", not a
    defect, and every bound below is built from it:
        U(out) = 2^-11 * sum over the 64-deep groups of max |term|  +  4e-6 * sum |terms|
    (second part: fp32 accumulation across blocks and the scale products).

  routing   pos is a bijection of the local slots onto the rows, rows are grouped by expert in
            expert order, sorted_tok inverts pos                                  (exact)
  stage 1   xq, xs == quant128(x) for every token that has a local slot            (exact)
  stage 2   with g, u the reference gate/up sums and dg = U(g), du = U(u), the kernel's value
            of a = silu(g) u is uncertain by da = 1.1 |u| dg + |silu(g)| du + 2e-5 |a| (fast
            exp, division); every group scale must be amax/448 within da(argmax)/448, every
            code a correct rounding of a/scale within da/scale
  stage 3   the down-projection rows and y against the reference applied to THE KERNEL'S OWN
            intermediate codes: |o - ref| <= U(o); |y - ref| <= 2^-8 |ref| (the one bf16
            rounding) + sum_k |w_k| U(o_k)
  end to end, from the inputs alone: stage 3 above feeds the kernel's codes to the reference's down
            projection (as input, never as an expected value).  Independently of that, the reference
            alone brackets y: every intermediate value lies within da of the reference's, so its
            group scale and code lie in an interval (rounding is monotone), so does the dequantized
            intermediate, and interval arithmetic through the down projection, U(o), the routing
            weights and the one bf16 rounding gives [y_lo, y_hi], which must contain the kernel's y.
            Most codes are pinned exactly; the few near a rounding boundary widen the bracket.
plus an end-to-end sanity net on all tokens (row-wise relative L2 error, exact zeros).
"""
import numpy as np
import pytest

import oracle
from paper_2604_18616_amd import inputs as I

pytestmark = pytest.mark.gpu
VALS = I.e4m3_values()
POS = VALS[:127]


def run(d, row_tile=0):
    import torch
    from paper_2604_18616_amd import binding
    t = {"x": torch.from_numpy(d["x"].view(np.int16)).view(torch.bfloat16).cuda()}
    for k in ("ids", "wts", "w13", "s13", "w2", "s2"):
        t[k] = torch.from_numpy(d[k]).cuda()
    T, H = d["x"].shape
    E, _, Isz = d["w2"].shape[0], None, d["w2"].shape[2]
    K = d["ids"].shape[1]
    y = torch.full((T, H), float("nan"), dtype=torch.bfloat16, device="cuda")
    need = binding.moe_workspace_bytes(T, H, Isz, E, K)
    ws = torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda")        # garbage: nothing may rely on zeros
    binding.moe_ffn_fp8(t["x"], t["ids"], t["wts"], t["w13"], t["s13"], t["w2"], t["s2"], y=y, workspace=ws, row_tile=row_tile)
    torch.cuda.synchronize()
    off = lambda part: binding.moe_workspace_offset(T, H, Isz, E, K, part)

    def part(idx, dtype, count):
        nbytes = count * np.dtype(dtype).itemsize
        return ws[off(idx):off(idx) + nbytes].cpu().numpy().view(dtype)

    slots = T * K
    offsets = part(0, np.int32, E + 1)
    A = int(offsets[E])
    out = dict(y=I.bf16_bits_to_f32(y.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64),
               offsets=offsets, sorted_tok=part(6, np.int32, slots)[:A], pos=part(7, np.int32, slots).reshape(T, K),
               xq=part(8, np.uint8, T * H).reshape(T, H), xs=part(9, np.float32, T * (H // 128)).reshape(T, H // 128),
               aq=part(10, np.uint8, max(A, 1) * Isz).reshape(-1, Isz)[:A],
               as_=part(11, np.float32, max(A, 1) * (Isz // 128)).reshape(-1, Isz // 128)[:A],
               o=part(12, np.float32, max(A, 1) * H).reshape(-1, H)[:A])
    return out


def spacing(v):
    """distance between neighbouring e4m3 values around magnitude v"""
    a = np.minimum(np.abs(v), 448.0)
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -6)))
    return 2.0 ** (e - 3)


def check_routing(w, d, g):
    ids, pos = d["ids"], g["pos"]
    local = (ids >= 0) & (ids < w.E)
    A = int(local.sum())
    assert int(g["offsets"][w.E]) == A and g["offsets"][0] == 0
    assert np.array_equal(np.diff(g["offsets"]), np.bincount(ids[local], minlength=w.E))
    assert np.all(pos[~local] == -1)
    assert sorted(pos[local].tolist()) == list(range(A))                        # bijection onto the rows
    tt, kk = np.nonzero(local)
    assert np.array_equal(g["sorted_tok"][pos[tt, kk]], tt)
    row_expert = np.searchsorted(g["offsets"][1:], np.arange(A), side="right")
    assert np.array_equal(row_expert[pos[tt, kk]], ids[tt, kk])                 # grouped by expert, in expert order


def check_stage1(w, d, g, tokens):
    xf = I.bf16_bits_to_f32(d["x"])
    for t in tokens:
        if not ((d["ids"][t] >= 0) & (d["ids"][t] < w.E)).any():
            continue                                   # never read by the products: the kernel skips them
        for b in range(w.H // 128):
            code, scale = oracle.quant_group(xf[t, 128 * b:128 * b + 128])
            assert np.array_equal(g["xq"][t, 128 * b:128 * b + 128], code), ("xq", t, b)
            assert g["xs"][t, b] == np.float32(scale), ("xs", t, b)


def mfma_uncertainty(act, wmat):
    """U(out) for out = wmat @ act (both dequantized, fp64): see the module docstring."""
    terms = np.abs(wmat * act[None, :])
    groups = terms.reshape(wmat.shape[0], -1, 64)
    return 2.0 ** -11 * groups.max(axis=2).sum(axis=1) + 4e-6 * terms.sum(axis=1)


def dequant_weights(codes, scales):
    return VALS[codes] * np.repeat(np.repeat(scales.astype(np.float64), 128, axis=0), 128, axis=1)


def check_slots(w, d, g, slots):
    """stages 2 and 3 for the listed (token, slot) pairs; returns reference rows and bounds keyed by (t, k)"""
    rows = {}
    for t, k in slots:
        e, r = int(d["ids"][t, k]), int(g["pos"][t, k])
        xf = I.bf16_bits_to_f32(d["x"][t])
        xd = np.concatenate([VALS[c] * float(sc) for c, sc in (oracle.quant_group(xf[128 * b:128 * b + 128]) for b in range(w.H // 128))])
        w13d = dequant_weights(d["w13"][e], d["s13"][e])
        gu, dgu = w13d @ xd, mfma_uncertainty(xd, w13d)
        gate, up, dg, du = gu[:w.I], gu[w.I:], dgu[:w.I], dgu[w.I:]
        silu = gate / (1.0 + np.exp(-gate))
        a = silu * up
        np.testing.assert_allclose(a, oracle.moe_intermediate(d["x"], d["w13"], d["s13"], t, e), rtol=1e-9, atol=1e-12)
        da = 1.1 * np.abs(up) * dg + np.abs(silu) * du + 2e-5 * np.abs(a)
        for b in range(w.I // 128):
            sl = slice(128 * b, 128 * b + 128)
            s = float(g["as_"][r, b])
            top = np.abs(a[sl]).argmax()
            assert abs(s - abs(a[sl][top]) / 448.0) <= (da[sl].max() + 1e-6 * abs(a[sl][top])) / 448.0 + 1e-30, \
                ("intermediate scale", t, k, b, s, abs(a[sl][top]) / 448.0)
            v = a[sl] / s
            c = VALS[g["aq"][r, sl]]
            assert not np.isnan(c).any()
            slack = 0.5 * np.maximum(spacing(v), spacing(c)) + da[sl] / s + 1e-6
            assert np.all(np.abs(c - np.clip(v, -448, 448)) <= slack), \
                ("intermediate code", t, k, b, float((np.abs(c - np.clip(v, -448, 448)) / slack).max()))
        o_ref = oracle.moe_down(g["aq"][r], g["as_"][r], d["w2"], d["s2"], e)
        deq = VALS[g["aq"][r]] * np.repeat(g["as_"][r].astype(np.float64), 128)
        do = mfma_uncertainty(deq, dequant_weights(d["w2"][e], d["s2"][e]))
        if ((d["ids"][t] >= 0) & (d["ids"][t] < w.E)).sum() > 1:   # the fp32 row exists only for tokens with several local slots: a single one goes straight to y (check_y)
            assert np.all(np.abs(g["o"][r] - o_ref) <= do + 1e-30), ("down row", t, k, float((np.abs(g["o"][r] - o_ref) / do).max()))
        rows[(t, k)] = (o_ref, do, a, da)
    return rows


GRID = np.unique(VALS[np.isfinite(VALS)])                 # the finite e4m3 values, ascending
MID = 0.5 * (GRID[1:] + GRID[:-1])


def bracket_y(w, d, t, rows):
    """[y_lo, y_hi] for token t from the inputs and the reference alone (see the module docstring); rows: check_slots' result"""
    y_lo, y_hi = np.zeros(w.H), np.zeros(w.H)
    for k in range(w.KTOP):
        if (t, k) not in rows:
            continue
        e = int(d["ids"][t, k])
        a, da = rows[(t, k)][2], rows[(t, k)][3]
        d_lo, d_hi = np.empty(w.I), np.empty(w.I)
        for b in range(w.I // 128):
            sl = slice(128 * b, 128 * b + 128)
            lo, hi = a[sl] - da[sl], a[sl] + da[sl]
            amax_lo = max(float(np.maximum(np.abs(a[sl]) - da[sl], 0.0).max()), 0.0)
            amax_hi = float((np.abs(a[sl]) + da[sl]).max())
            if amax_hi == 0.0:
                s_lo = s_hi = 1.0
            else:
                s_lo, s_hi = amax_lo / 448.0 * (1 - 2e-6), amax_hi / 448.0 * (1 + 2e-6)
                s_lo = max(s_lo, 1e-300)
            v_lo = np.minimum(lo / s_lo, lo / s_hi)
            v_hi = np.maximum(hi / s_lo, hi / s_hi)
            v_lo = np.clip(v_lo - 2e-6 * np.abs(v_lo), -448, 448)
            v_hi = np.clip(v_hi + 2e-6 * np.abs(v_hi), -448, 448)
            c_lo = GRID[np.searchsorted(MID, v_lo, side="left")]       # rounding is monotone; ties resolved outwards
            c_hi = GRID[np.searchsorted(MID, v_hi, side="right")]
            d_lo[sl] = np.minimum(c_lo * s_lo, c_lo * s_hi)
            d_hi[sl] = np.maximum(c_hi * s_lo, c_hi * s_hi)
        w2d = dequant_weights(d["w2"][e], d["s2"][e])
        wp, wn = np.maximum(w2d, 0.0), np.minimum(w2d, 0.0)
        o_lo, o_hi = wp @ d_lo + wn @ d_hi, wp @ d_hi + wn @ d_lo
        u = mfma_uncertainty(np.maximum(np.abs(d_lo), np.abs(d_hi)), w2d)
        wt = float(d["wts"][t, k])
        lo_k, hi_k = wt * (o_lo - u), wt * (o_hi + u)
        y_lo += np.minimum(lo_k, hi_k)
        y_hi += np.maximum(lo_k, hi_k)
    r = 2.0 ** -8 * np.maximum(np.abs(y_lo), np.abs(y_hi)) + 1e-30
    return y_lo - r, y_hi + r


def check_y_from_inputs_alone(w, d, g, tokens, rows):
    widths = []
    for t in tokens:
        if not any((t, k) in rows for k in range(w.KTOP)):
            continue
        y_lo, y_hi = bracket_y(w, d, t, rows)
        y = g["y"][t]
        assert np.all((y >= y_lo) & (y <= y_hi)), ("y outside the reference's bracket", t, float(np.max(np.maximum(y_lo - y, y - y_hi))))
        ref = oracle.moe_ref(**d, rows=[t])[0]
        assert np.all((ref >= y_lo) & (ref <= y_hi)), ("the reference's own y outside its bracket", t)
        widths.append(float(np.median((y_hi - y_lo) / (np.abs(ref) + 1e-30))))
    return widths


def check_y(w, d, g, tokens):
    slots = [(t, k) for t in tokens for k in range(w.KTOP) if 0 <= d["ids"][t, k] < w.E]
    rows = check_slots(w, d, g, slots)
    widths = check_y_from_inputs_alone(w, d, g, tokens, rows)
    if widths:
        print("y bracket from the inputs alone: median relative width %.3g (median over %d tokens)" % (float(np.median(widths)), len(widths)), flush=True)
    for t in tokens:
        y_ref, s_abs = np.zeros(w.H), np.zeros(w.H)
        for k in range(w.KTOP):
            if (t, k) in rows:
                y_ref += float(d["wts"][t, k]) * rows[(t, k)][0]
                s_abs += abs(float(d["wts"][t, k])) * rows[(t, k)][1]
        err = np.abs(g["y"][t] - y_ref)
        assert np.all(err <= 2.0 ** -8 * np.abs(y_ref) + s_abs + 1e-30), ("y", t, float(err.max()))


def sanity_net(y, ref, what):
    assert np.isfinite(y).all(), what
    zero = ~ref.any(axis=1)
    assert not y[zero].any(), what + ": rows without a local expert must be exactly zero"
    live = ~zero
    if live.any():
        rel = np.sqrt(((y - ref)[live] ** 2).sum(axis=1) / (ref[live] ** 2).sum(axis=1))
        assert rel.max() < 0.06 and np.median(rel) < 5e-3, (what, float(rel.max()), float(np.median(rel)))


SMALL = [dict(T=12), dict(T=64, EP=1), dict(T=200, H=384, I=256, E=3, KTOP=3, EP=1), dict(T=70, H=128, I=128, E=2, KTOP=1, EP=1),
         dict(T=300, H=512, I=384, E=8, KTOP=4, EP=2), dict(T=1, H=256, I=128, E=4, KTOP=2, EP=1), dict(T=9, EP=16),
         dict(T=300, H=128, I=128, E=256, KTOP=16, EP=1),          # the largest expert and slot counts the library takes
         dict(T=128, H=128, I=256, E=1, KTOP=1, EP=1),              # one expert, exactly full row tiles
         dict(T=40, H=256, I=16384, E=2, KTOP=1, EP=1),             # the longest reduction of the down product the library takes
         dict(T=24, H=16384, I=128, E=2, KTOP=2, EP=1)]             # and of the gate/up product


@pytest.mark.parametrize("row_tile", [64, 128])
@pytest.mark.parametrize("cfg", SMALL)
def test_small_configurations(cfg, row_tile):
    c = dict(H=256, I=128, E=4, KTOP=2, EP=2)
    c.update(cfg)
    T = c.pop("T")
    w = I.MoeWorkload("t", T, 40 + T, **c)
    d = I.make_moe(w)
    print("moe case", w, "local slots", w.local_slots(d["ids"]), "row tile", row_tile, flush=True)
    g = run(d, row_tile)
    check_routing(w, d, g)
    tokens = list(range(min(T, 24))) + ([T - 1] if T > 24 else [])
    check_stage1(w, d, g, tokens)
    check_y(w, d, g, tokens)
    sanity_net(g["y"], oracle.moe_ref(**d), str(w))


# every token goes to both experts, so an expert has T rows.  With 128-row tiles: 700 = 5 x 128 + 60 (a 64-row tail),
# 300 = 128 + 128 + 44, 280 = 128 + 128 + 24, 150 and 160 (one tile on the 160-row code, 160 being its limit),
# 161 = 128 + 33 (one row too many for a single tile).  With 64-row tiles the same sizes give up to 11 tiles.
@pytest.mark.parametrize("row_tile", [64, 128])
@pytest.mark.parametrize("T", [700, 300, 280, 150, 160, 161, 90, 96, 97])
def test_many_rows_per_expert_span_several_row_tiles(T, row_tile):
    w = I.MoeWorkload("t", T, 77 + T, H=256, I=256, E=2, KTOP=2, EP=1)
    d = I.make_moe(w)
    print("moe case", w, "row tile", row_tile, flush=True)
    g = run(d, row_tile)
    check_routing(w, d, g)
    tokens = sorted({t for t in (0, 1, 63, 64, 65, 127, 128, 129, 149, 255, 256, 257, T - 45, T - 2, T - 1) if 0 <= t < T})
    check_stage1(w, d, g, tokens)
    check_y(w, d, g, tokens)
    sanity_net(g["y"], oracle.moe_ref(**d), str(w))


def test_no_local_expert_at_all():
    w = I.MoeWorkload("t", 33, 5, H=256, I=128, E=4, KTOP=2, EP=1)
    d = I.make_moe(w)
    d["ids"] = np.full_like(d["ids"], -1)
    g = run(d)
    assert not g["y"].any() and int(g["offsets"][w.E]) == 0 and np.all(g["pos"] == -1)


# M1024: about 16 rows per expert (the 64-row code); M8192: 128 +- 11 rows per expert, so that the 64-, 128- and
# 160-row codes all run at the paper's H and I in one call
@pytest.mark.parametrize("name,row_tile", [("M1024", 0), ("M1024", 64), ("M8192", 0)])
def test_paper_shape_on_sampled_tokens(name, row_tile):
    w = I.MOE_WORKLOADS[name]
    d = I.make_moe(w)
    print("moe workload", w, "local slots", w.local_slots(d["ids"]), "row tile", row_tile, flush=True)
    g = run(d, row_tile)
    check_routing(w, d, g)
    tokens = I.sample_tokens(w, d["ids"], 12).tolist()
    check_stage1(w, d, g, tokens)
    check_y(w, d, g, tokens)
    assert not g["y"][~(d["ids"] >= 0).any(axis=1)].any()
