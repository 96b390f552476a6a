"""moe_ffn_fp8_static, the entry point for callers that cannot allocate: its scratch memory is a device array
inside the library.  Called through the C ABI twice in a row on one GPU -- a problem that nearly fills the array,
then a smaller one on top of what the first left there -- and compared bit for bit with moe_ffn_fp8 on a
caller-owned workspace (the same kernels run, and the result does not depend on the row order the routing
happens to produce); a third, tiny call is also held against the CPU reference."""
import numpy as np
import pytest

from paper_2604_18616_amd import inputs as I

pytestmark = pytest.mark.gpu


def device_inputs(w):
    import torch
    d = I.make_moe(w)
    t = {"x": torch.from_numpy(d["x"].view(np.int16)).view(torch.bfloat16).cuda()}
    for k in ("ids", "wts", "w13", "s13", "w2", "s2"):
        t[k] = torch.from_numpy(d[k]).cuda()
    return d, t


def both_ways(lib, w, t):
    """y of moe_ffn_fp8_static and of moe_ffn_fp8 (garbage-filled workspace), as int16 bit patterns on the host."""
    import torch
    sp = torch.cuda.current_stream().cuda_stream
    argv = (t["x"].data_ptr(), t["ids"].data_ptr(), t["wts"].data_ptr(), t["w13"].data_ptr(), t["s13"].data_ptr(),
            t["w2"].data_ptr(), t["s2"].data_ptr())
    dims = (w.T, w.H, w.I, w.E, w.KTOP)
    y_static = torch.full((w.T, w.H), float("nan"), dtype=torch.bfloat16, device="cuda")
    print("moe_ffn_fp8_static", dims, flush=True)
    rc = lib.moe_ffn_fp8_static(*argv, y_static.data_ptr(), *dims, sp)
    assert rc == 0, rc
    torch.cuda.synchronize()
    need = lib.moe_ffn_fp8_workspace_bytes(*dims)
    ws = torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda")
    y_ws = torch.full((w.T, w.H), float("nan"), dtype=torch.bfloat16, device="cuda")
    rc = lib.moe_ffn_fp8(*argv, y_ws.data_ptr(), *dims, ws.data_ptr(), need, sp)
    assert rc == 0, rc
    torch.cuda.synchronize()
    return y_static.view(torch.int16).cpu().numpy(), y_ws.view(torch.int16).cpu().numpy(), need


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    from paper_2604_18616_amd import binding
    import oracle
    lib = binding.load_library()
    limit = 128 << 20
    # 1: close to the capacity (many tokens, small experts); 2: a smaller problem of another shape right after it
    big = I.MoeWorkload("static_big", 26000, 61, H=256, I=128, E=4, KTOP=4, EP=1)
    small = I.MoeWorkload("static_small", 333, 62, H=512, I=256, E=8, KTOP=2, EP=2)
    for w in (big, small):
        d, t = device_inputs(w)
        ys, yw, need = both_ways(lib, w, t)
        assert need <= limit and (w is small or need > limit * 0.85), need
        assert not np.isnan(I.bf16_bits_to_f32(ys.view(np.uint16))).any()
        assert np.array_equal(ys, yw), (w.name, int((ys != yw).sum()))
    # the smaller call once more against the CPU reference (the end-to-end net of the parity tests)
    y = I.bf16_bits_to_f32(ys.view(np.uint16)).astype(np.float64)
    rows = I.sample_tokens(small, d["ids"], 24)
    ref = oracle.moe_ref(rows=rows, **d)
    live = ref.any(axis=1)
    rel = np.sqrt(((y[rows] - ref)[live] ** 2).sum(axis=1) / (ref[live] ** 2).sum(axis=1))
    assert not y[rows][~live].any() and rel.max() < 0.06 and np.median(rel) < 5e-3, (rel.max(), np.median(rel))
    # beyond the capacity: refused, nothing launched
    import torch
    a = torch.zeros(64, dtype=torch.uint8, device="cuda").data_ptr()
    assert lib.moe_ffn_fp8_static(a, a, a, a, a, a, a, a, 1032, 7168, 2048, 32, 4, None) == -7
