"""Weights handed over as the bf16 GEMMs read them ([out, in], q | k | v in one matrix): the stage multiplies by the
caller's memory, keeps no second copy, and computes what the [in, out] hand-over computes (Sec. 2: device j holds
the chunk E_theta_j once; Table 1 counts the model memory once per device)."""
import numpy as np
import pytest
import torch

from paper_2505_21070_amd import synth
from tests.harness import check, oracle_stage, to_dev, to_np

pytestmark = pytest.mark.gpu

CASES = [
    ("small_bf16", dict(ffn_dim=768)),      # ragged token counts, head_dim 128, text MLP (text_dim != dim)
    ("wide128_bf16", {}),                   # 256 x 256 GEMM tiles, per-head q|k|v epilogue, 256-query attention blocks
    ("wide64_bf16", {}),                    # head_dim 64
]


@pytest.mark.parametrize("name,over", CASES, ids=[c[0] for c in CASES])
def test_out_in_weights_same_bits_as_in_out_and_match_the_oracle(name, over, progress):
    from paper_2505_21070_amd import binding as B
    cfg, w, text, blocks = synth.make_case(name, seed=11, **over)
    nf, nc = cfg["block_frames"], cfg["cache_frames"]
    wd = B.weights_to_device(w, "bf16")
    td = to_dev(text, cfg)
    conf_io = B.make_config(cfg, debug_taps=1, max_abs_frames=64)
    conf_oi = B.make_config(cfg, debug_taps=1, max_abs_frames=64, weight_layout="out_in")
    # the workspace no longer holds the matrices: 3 D^2 (q|k|v) + 3 D^2 (o, cross q, cross o) + 2 D F per layer
    D, F = cfg["dim"], cfg["ffn_dim"]
    held = cfg["n_layers"] * (6 * D * D + 2 * D * F) * 2
    assert B.workspace_bytes(conf_io) - B.workspace_bytes(conf_oi) >= held
    a = B.Stage(conf_io, wd, td)
    b = B.Stage(conf_oi, B.weights_out_in(wd), td)
    o = oracle_stage(cfg, w, text)
    progress("stages built")
    outs = []
    for g in (a, b):
        y0 = g.forward(to_dev(blocks[0], cfg), nf, nf, 700.0)
        g.cache_update(0, nc)
        y1 = g.forward(to_dev(blocks[1], cfg), nf, 0, 650.0)
        li = cfg["n_layers"] - 1
        outs.append([y0, y1] + [g.peek(what, li) for what in ("k", "v", "text_k", "text_v", "attn", "cross_attn", "x_res")])
    torch.cuda.synchronize()
    for ta, tb in zip(*outs):
        assert torch.equal(ta, tb)
    progress("both layouts agree bit for bit")
    o.forward(blocks[0].numpy(), nf, nf, 700.0)
    o.cache_update(0, nc)
    r = o.forward(blocks[1].numpy(), nf, 0, 650.0)
    check(f"{name}/out_in/x_out", to_np(outs[1][1]), r, "bf16")
    # what the layers added, from the fp32 residual stream (the rounding of x_out to bf16 would swamp it)
    check(f"{name}/out_in/delta", to_np(outs[1][-1]) - blocks[1].numpy().astype(np.float64), r - blocks[1].numpy(), "bf16")


def test_out_in_rejects_matrices_that_are_not_one_qkv_block():
    from paper_2505_21070_amd import binding as B
    cfg, w, text, _ = synth.make_case("wide128_bf16", seed=3)
    wd = B.weights_out_in(B.weights_to_device(w, "bf16"))
    wd["layers"][0]["wk"] = wd["layers"][0]["wk"].clone()          # same values, but no longer behind wq in memory
    conf = B.make_config(cfg, weight_layout="out_in")
    with pytest.raises(B.DualParalError) as ei:
        B.Stage(conf, wd, to_dev(text, cfg))
    assert ei.value.code == B.DP_EINVAL and "back to back" in str(ei.value)
