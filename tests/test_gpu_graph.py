"""The library launches kernels on the caller's stream and nothing else (no allocation, no
memset, no synchronisation), so a training step or a decode call can be captured in a HIP
graph.  Replays are checked against the eager results, with eager work between them."""
import pytest
import torch

from helpers import dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sb():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2410_17980_amd import binding
    binding.load(build_if_missing=False)
    return binding


@pytest.fixture(scope="module")
def gen():
    from paper_2410_17980_amd import inputs
    return inputs


def test_training_step_in_a_graph(sb, gen):
    B, H, T, d = 2, 4, 700, 128
    q, k, v, g = dev(*gen.gaussian(B, H, T, d, seed=1, sharp_half=True, with_dout=True))
    r = gen.remainder_embedding(H, d, seed=2).cuda()
    o = torch.empty_like(q)
    m = torch.empty(B, H, T, dtype=torch.float32, device="cuda")
    dq, dk, dv = (torch.empty(B, H, T, d, dtype=torch.float32, device="cuda") for _ in range(3))
    dr = torch.empty(H, d, dtype=torch.float32, device="cuda")
    ws = torch.empty(sb.sb_attn_bwd_workspace_bytes(B, H, T, d), dtype=torch.uint8, device="cuda")

    def step():
        sb.sb_attn_fwd_rb(q, k, v, r, o=o, m=m)
        sb.sb_attn_bwd_rb(q, k, v, r, m, g, dq=dq, dk=dk, dv=dv, dr=dr, workspace=ws)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (o, m, dq, dk, dv, dr)]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for rep in range(3):
        for t in (o, m, dq, dk, dv, dr):
            t.fill_(float("nan") if t.is_floating_point() else 0)
        ws.random_(0, 255)                       # the workspace's previous contents must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("o", "m", "dq", "dk", "dv", "dr"), (o, m, dq, dk, dv, dr), want):
            assert torch.equal(a, b), f"replay {rep}: {name} differs from the eager result"
        sb.sb_attn_fwd(q, k, v)                  # eager work between the replays
        torch.cuda.synchronize()


def test_decode_in_a_graph(sb, gen):
    B, H, Hkv, T, d = 2, 8, 2, 3000, 128
    q, _, _ = gen.gaussian(B, H, 1, d, seed=3)
    _, k, v = gen.gaussian(B, Hkv, T, d, seed=4)
    q, k, v = dev(q[:, :, 0].contiguous(), k, v)
    o = torch.empty_like(q)
    ws = torch.empty(sb.load().sb_attn_decode_workspace_bytes(B, H, T, d), dtype=torch.uint8, device="cuda")
    sb.sb_attn_decode(q, k, v, o=o, workspace=ws)
    torch.cuda.synchronize()
    want = o.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        sb.sb_attn_decode(q, k, v, o=o, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        sb.sb_attn_decode(q, k, v, o=o, workspace=ws)
    for rep in range(3):
        o.zero_()
        ws.random_(0, 255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o, want), f"replay {rep}"
