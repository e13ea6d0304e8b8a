"""dp_head_forward_static (the output head for callers that cannot allocate: its scratch is a device array
inside the library) against dp_head_forward, whose result it must reproduce bit for bit: two calls in a row,
the second with a smaller input, so that what the first call left in the array cannot leak into the second."""
import pytest
import torch

from paper_2505_21070_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,channels,frames", [("tiny", 4, 3), ("small_bf16", 16, 3), ("tiny_bf16", 16, 2)])
def test_static_head_matches_workspace_head(name, channels, frames):
    from paper_2505_21070_amd import binding as B
    cfg = synth.stage_config(name)
    w = synth.make_weights(cfg, seed=31)
    td = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    dev = {k: v.to("cuda", td).contiguous() for k, v in synth.make_end_weights(cfg, channels, 31).items()}
    dev.update({k: w["stage"][k].to("cuda", td).contiguous() for k in ("wt1", "bt1", "wt2", "bt2")})
    ends = B.Ends(cfg, dev, channels, frames)
    gen = torch.Generator().manual_seed(32)
    tok = cfg["tok_h"] * cfg["tok_w"]
    x_big = synth.make_block(cfg, frames, gen).to("cuda", td).contiguous()
    x_small = synth.make_block(cfg, 1, gen).to("cuda", td).contiguous()
    shape = lambda n: (n, 2 * cfg["tok_h"], 2 * cfg["tok_w"], channels)
    out_big = torch.full(shape(frames), float("nan"), device="cuda")
    out_small = torch.full(shape(1), float("nan"), device="cuda")
    ref_big = ends.head(x_big, 437.0, frames)
    ref_small = ends.head(x_small, 812.0, 1)
    torch.cuda.synchronize()
    B.head_forward_static(cfg, dev, channels, x_big, 437.0, frames, out_big)        # first call
    B.head_forward_static(cfg, dev, channels, x_small, 812.0, 1, out_small)         # second call, smaller input
    torch.cuda.synchronize()
    assert torch.isfinite(ref_big).all() and ref_big.abs().max() > 0
    assert torch.equal(out_big, ref_big)
    assert torch.equal(out_small, ref_small)
    assert not torch.equal(ref_small, ref_big[:1])


def test_static_head_rejects_what_does_not_fit():
    from paper_2505_21070_amd import binding as B
    cfg = synth.stage_config("wan1p3b_stage")
    td = torch.bfloat16
    w = synth.make_weights(dict(cfg, n_layers=0), seed=33)       # stage-level weights only
    dev = {k: v.to("cuda", td).contiguous() for k, v in synth.make_end_weights(cfg, 16, 33).items()}
    dev.update({k: w["stage"][k].to("cuda", td).contiguous() for k in ("wt1", "bt1", "wt2", "bt2")})
    tok = cfg["tok_h"] * cfg["tok_w"]
    x = torch.zeros((5 * tok, cfg["dim"]), dtype=td, device="cuda")
    out = torch.zeros((5, 2 * cfg["tok_h"], 2 * cfg["tok_w"], 16), device="cuda")
    with pytest.raises(B.DualParalError) as ei:
        B.head_forward_static(cfg, dev, 16, x, 500.0, 5, out)                       # 7800 tokens: 75 MB > 64 MiB
    assert ei.value.code == B.DP_ENOMEM and "64 MiB" in str(ei.value)
    one = torch.full((1, 2 * cfg["tok_h"], 2 * cfg["tok_w"], 16), float("nan"), device="cuda")
    B.head_forward_static(cfg, dev, 16, x[:tok].contiguous(), 500.0, 1, one)        # one frame fits
    torch.cuda.synchronize()
    assert torch.isfinite(one).all()
