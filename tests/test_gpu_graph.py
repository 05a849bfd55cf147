"""The layer as a HIP graph: its five launches are recorded once and replayed on new inputs.
Every replay is checked bit for bit against an eager run, with eager work and synchronisations
between the replays (the entry points allocate nothing and record no memset nodes)."""
import pytest
import torch

from paper_2512_24086_amd import inputs
from tests import helpers as hp

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("over", [dict(), dict(block=64, block_k=128), dict(cdf_threshold=0.8)],
                         ids=["topn", "rect", "cdf"])
def test_layer_replays_from_a_graph(over):
    wl = inputs.Workload("graph", 23, 1, 3, 128, 5, 10, 13, 128, 0.5, 1, 0.3, text_tokens=17)
    if "block" in over:
        import dataclasses
        over = dict(over)
        wl = dataclasses.replace(wl, block=over.pop("block"))
    plan = hp.make_plan(wl, **over)
    base = [x.to(DEV) for x in inputs.make_qkv(wl)]
    q, k, v = (x.clone() for x in base)                       # static input buffers of the graph
    buf, buf_eager = plan.alloc(DEV), plan.alloc(DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        plan.layer_fused(q, k, v, buf)                         # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        plan.layer_fused(q, k, v, buf)
    for rep in range(4):
        # eager work between the replays: new inputs (a rotation of the heads and a sign flip)
        for dst, src in zip((q, k, v), base):
            dst.copy_(torch.roll(src, rep, dims=1) * (-1.0 if rep % 2 else 1.0))
        buf["o"].fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        plan.layer_fused(q, k, v, buf_eager)
        torch.cuda.synchronize()
        assert torch.isfinite(buf["o"].float()).all()
        assert torch.equal(buf["o"].view(torch.int16), buf_eager["o"].view(torch.int16)), rep
        assert torch.equal(buf["blk_cnt"], buf_eager["blk_cnt"])
        if "cdf_threshold" not in over:          # (entries past a row's count are unspecified in that mode)
            assert torch.equal(buf["blk_idx"], buf_eager["blk_idx"])
    plan.close()
