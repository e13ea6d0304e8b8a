"""dp_stage_forward under HIP graph capture: the call allocates nothing, synchronises nothing and records no
memset node, so a serving loop can capture it.  A captured forward is replayed several times with eager work on
the same stage in between and must give the eager results bit for bit."""
import pytest
import torch

from harness import gpu_stage, to_dev
from paper_2505_21070_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["tiny", "tiny_bf16", "wide128_bf16"])
def test_captured_forward_replays_bit_exact(name):
    cfg, w, text, blocks = synth.make_case(name, seed=3, strong_gate=True)
    nf, nc = cfg["block_frames"], cfg["cache_frames"]
    g = gpu_stage(cfg, w, text)
    x0, x1 = to_dev(blocks[0], cfg), to_dev(blocks[1], cfg)
    x2 = (x1.float() * 0.5 + 0.1).to(x1.dtype)
    g.forward(x0, nf, nf, 625.0)
    g.cache_update(0, nc)                          # from here on the stage's host state stays as it is
    y1 = g.forward(x1, nf, 0, 500.0).clone()
    y2 = g.forward(x2, nf, 0, 500.0).clone()
    torch.cuda.synchronize()
    xs, ys = x1.clone(), torch.empty_like(y1)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        g.forward(xs, nf, 0, 500.0, out=ys)        # first use of every kernel happens outside the capture
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        g.forward(xs, nf, 0, 500.0, out=ys)
    for rep in range(3):
        xs.copy_(x1)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ys, y1), f"replay {rep}, first input"
        assert torch.equal(g.forward(x2, nf, 0, 500.0), y2)      # eager work on the same stage in between
        torch.cuda.synchronize()
        xs.copy_(x2)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ys, y2), f"replay {rep}, second input"
