"""The three entry points under HIP graph capture: the library allocates nothing, synchronises
nothing and records no memset nodes, so a captured call must replay to the same bits as the
eager call, on every replay, with other work in between."""
import numpy as np
import pytest

from paper_2604_18616_amd import inputs as I

pytestmark = pytest.mark.gpu


def dev_bf16(bits):
    import torch
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()


def test_captured_calls_replay_to_the_eager_bits():
    import torch
    from paper_2604_18616_amd import binding

    aw = I.Workload("g", 2, 4, 2, 300, 333, 128, True, 21)
    q, k, v = (dev_bf16(x) for x in I.make_qkv(aw))
    gw = I.GemmWorkload("g", 520, 264, 200, 22)
    a, b = (dev_bf16(x) for x in I.make_ab(gw))
    mw = I.MoeWorkload("g", 150, 23, H=256, I=256, E=4, KTOP=2, EP=2)
    md = I.make_moe(mw)
    mt = {key: (dev_bf16(val) if key == "x" else torch.from_numpy(val).cuda()) for key, val in md.items()}
    ws = torch.empty(binding.moe_workspace_bytes(mw.T, mw.H, mw.I, mw.E, mw.KTOP), dtype=torch.uint8, device="cuda")

    def outputs():
        return (torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device="cuda"),
                torch.full(q.shape[:3], float("nan"), dtype=torch.float32, device="cuda"),
                torch.full((gw.M, gw.N), float("nan"), dtype=torch.bfloat16, device="cuda"),
                torch.full((mw.T, mw.H), float("nan"), dtype=torch.bfloat16, device="cuda"))

    def run_all(o, lse, c, y):
        binding.attn_fwd(q, k, v, o, lse, causal=True, scale=aw.scale)
        binding.gemm_bf16(a, b, c)
        binding.moe_ffn_fp8(mt["x"], mt["ids"], mt["wts"], mt["w13"], mt["s13"], mt["w2"], mt["s2"], y=y, workspace=ws)

    eager = outputs()
    run_all(*eager)
    torch.cuda.synchronize()
    want = [t.clone() for t in eager]

    cap = outputs()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        run_all(*cap)                      # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run_all(*cap)
    torch.cuda.synchronize()
    for replay in range(3):
        for t in cap:
            t.fill_(float("nan"))          # a small fill kernel, not a memset node
        ws.fill_(0xFF)
        torch.cuda.synchronize()
        graph.replay()
        scratch = torch.randn(1 << 20, device="cuda").sum()     # the program's own eager work between replays
        torch.cuda.synchronize()
        for got, ref in zip(cap, want):
            assert torch.equal(got.view(torch.int16 if got.dtype == torch.bfloat16 else torch.int32),
                               ref.view(torch.int16 if ref.dtype == torch.bfloat16 else torch.int32)), replay
        assert torch.isfinite(scratch)
