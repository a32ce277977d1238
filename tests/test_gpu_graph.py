"""Both entry points under HIP graph capture: they allocate nothing, clear nothing and never
synchronise, so a caller can record them into a graph.  A graph is replayed several times,
with the program's own eager work and synchronisations in between, and every replay is compared
with the eager result bit for bit."""
import pytest

from paper_2403_16863_amd import inputs as I

pytestmark = pytest.mark.gpu


def test_attention_and_gemm_replay_from_a_graph():
    import torch
    import paper_2403_16863_amd as A
    from paper_2403_16863_amd import gemm
    from tests.gpu_util import to_device
    w = I.Workload("g", 2, 4, 700, 128, True, I.BF16)
    qb, kb, vb = I.make_qkv(w, seed=1)
    q, k, v = (to_device(x, w.dtype) for x in (qb, kb, vb))
    out, lse = torch.empty_like(q), torch.empty(q.shape[:3], dtype=torch.float32, device="cuda")
    ab, bb = I.make_gemm(200, 136, 520, I.F16, seed=2)
    a, b = to_device(ab, I.F16), to_device(bb, I.F16)
    c = torch.empty((200, 136), dtype=torch.float16, device="cuda")

    A.attn_fwd(q, k, v, out, lse, True, w.scale)
    gemm.gemm_lrelu(a, b, c, 0.01)
    torch.cuda.synchronize()
    want = (out.clone(), lse.clone(), c.clone())

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            A.attn_fwd(q, k, v, out, lse, True, w.scale, stream=side.cuda_stream)
            gemm.gemm_lrelu(a, b, c, 0.01, stream=side.cuda_stream)
    torch.cuda.synchronize()
    for rep in range(4):
        out.fill_(float("nan"))
        lse.fill_(float("nan"))
        c.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), want[0].view(torch.int16)), f"replay {rep}: O"
        assert torch.equal(lse, want[1]), f"replay {rep}: lse"
        assert torch.equal(c.view(torch.int16), want[2].view(torch.int16)), f"replay {rep}: C"
        # eager work between replays
        A.attn_fwd(q, k, v, out, lse, True, w.scale)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), want[0].view(torch.int16))
