"""GPU parity of the model's ends (patch embedding, output head) and the Euler scheduler step against the
oracle, and the whole latent-space loop latent -> tokens -> stage -> velocity -> updated latent."""
import numpy as np
import pytest
import torch

from harness import check, gpu_stage, oracle_stage, to_dev, to_np
from oracle.ends import OracleEnds, euler_step
from paper_2505_21070_amd import synth

pytestmark = pytest.mark.gpu


def make_ends(cfg, w, channels, max_frames, seed=0):
    from paper_2505_21070_amd import binding as B
    ew = synth.make_end_weights(cfg, channels, seed)
    host = {k: v.numpy() for k, v in ew.items()}
    host.update({k: w["stage"][k].numpy() for k in ("wt1", "bt1", "wt2", "bt2")})
    td = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    dev = {k: torch.from_numpy(v).to(device="cuda", dtype=td).contiguous() for k, v in host.items()}
    return B.Ends(cfg, dev, channels, max_frames), OracleEnds(dict(cfg, channels=channels), host)


@pytest.mark.parametrize("name,channels,frames", [("tiny", 4, 2), ("tiny", 16, 3), ("small_bf16", 16, 3), ("tiny_bf16", 16, 2)])
def test_embed_and_head_match_oracle(name, channels, frames):
    cfg = synth.stage_config(name)
    w = synth.make_weights(cfg, seed=1)
    g, o = make_ends(cfg, w, channels, frames, seed=1)
    gen = torch.Generator().manual_seed(2)
    lat = synth.make_latent(cfg, frames, channels, gen)
    x = g.embed(lat.cuda())
    check(f"{name}/embed", to_np(x), o.embed(lat.numpy().astype(np.float64)), cfg["dtype"])
    tokens = synth.make_block(cfg, frames, gen)
    v = g.head(to_dev(tokens, cfg), 437.0, frames)
    ref = o.head(tokens.numpy().astype(np.float64), 437.0, frames)
    assert v.shape == ref.shape
    check(f"{name}/head", to_np(v).reshape(-1, channels), ref.reshape(-1, channels), cfg["dtype"])
    # fewer frames than the handle was sized for
    v1 = g.head(to_dev(tokens, cfg)[: g.tok].contiguous(), 437.0, 1)
    check(f"{name}/head1", to_np(v1).reshape(-1, channels), ref[:1].reshape(-1, channels), cfg["dtype"])


def test_embed_and_head_at_wan_shape_sampled_rows():
    cfg = synth.stage_config("wan1p3b_stage")
    w = synth.make_weights(cfg, seed=3)
    frames, C = 4, 16
    g, o = make_ends(cfg, w, C, frames, seed=3)
    gen = torch.Generator().manual_seed(4)
    lat = synth.make_latent(cfg, frames, C, gen)
    x = g.embed(lat.cuda())
    ref = o.embed(lat.numpy().astype(np.float64))
    rows = np.r_[0:64, 3000:3064, ref.shape[0] - 64:ref.shape[0]]
    check("wan/embed", to_np(x)[rows], ref[rows], "bf16")
    tokens = synth.make_block(cfg, frames, gen)
    v = g.head(to_dev(tokens, cfg), 250.0, frames)
    vref = o.head(tokens.numpy().astype(np.float64), 250.0, frames)
    check("wan/head", to_np(v).reshape(-1, C), vref.reshape(-1, C), "bf16")


def test_euler_step_and_error_paths():
    from paper_2505_21070_amd import binding as B
    gen = torch.Generator().manual_seed(5)
    x = torch.randn(1000003, generator=gen)           # odd length
    v = torch.randn(1000003, generator=gen)
    xd = x.cuda()
    B.euler_step(xd, v.cuda(), 0.5, 0.375)
    ref = euler_step(x.numpy(), v.numpy(), np.float32(0.5), np.float32(0.375))
    assert np.abs(xd.cpu().numpy() - ref).max() <= 1e-6
    B.euler_step(xd[:0], v.cuda()[:0], 0.5, 0.25)     # empty: no-op
    cfg = synth.stage_config("tiny")
    w = synth.make_weights(cfg, seed=1)
    g, _ = make_ends(cfg, w, 4, 2)
    with pytest.raises(B.DualParalError) as ei:
        g.head(torch.zeros((3 * g.tok, cfg["dim"]), device="cuda"), 1.0, 3)      # more frames than max_frames
    assert ei.value.code == B.DP_EINVAL
    cfg16 = synth.stage_config("tiny_bf16")
    with pytest.raises(B.DualParalError) as ei:       # bf16 needs 4 * channels % 64 == 0
        make_ends(cfg16, synth.make_weights(cfg16, seed=1), 3, 2)
    assert ei.value.code == B.DP_EINVAL
    torch.cuda.synchronize()


def test_latent_space_denoising_loop_matches_oracle():
    """latent --embed--> tokens --stage--> tokens --head--> velocity --Euler--> latent, three levels, one block with
    a cached neighbour; the same chain on the oracle (fp32 configuration, so errors stay at rounding level)."""
    from paper_2505_21070_amd import binding as B
    cfg, w, text, _ = synth.make_case("tiny", seed=6, strong_gate=True)
    C, nf, nc, T = 4, cfg["block_frames"], cfg["cache_frames"], 3
    g_ends, o_ends = make_ends(cfg, w, C, nf, seed=6)
    g, o = gpu_stage(cfg, w, text, max_abs_frames=16), oracle_stage(cfg, w, text)
    gen = torch.Generator().manual_seed(7)
    lat_nb, lat = synth.make_latent(cfg, nf, C, gen), synth.make_latent(cfg, nf, C, gen)
    xg, xo = lat.cuda().clone(), lat.numpy().astype(np.float64)
    for k in range(T, 0, -1):
        t, t_nb = 1000.0 * k / T, 1000.0 * min(k + 1, T) / T
        # the neighbour (later block, one level noisier) runs first and leaves its first frames' K/V behind
        g.forward(g_ends.embed(lat_nb.cuda()), nf, nf, t_nb); g.cache_update(0, nc)
        o.forward(o_ends.embed(lat_nb.numpy().astype(np.float64)), nf, nf, t_nb); o.cache_update(0, nc)
        vg = g_ends.head(g.forward(g_ends.embed(xg), nf, 0, t), t, nf)
        vo = o_ends.head(o.forward(o_ends.embed(xo), nf, 0, t), t, nf)
        check(f"loop/v{k}", to_np(vg).reshape(-1, C), vo.reshape(-1, C), "f32")
        B.euler_step(xg, vg, k / T, (k - 1) / T)
        xo = euler_step(xo, vo, k / T, (k - 1) / T)
        check(f"loop/x{k}", to_np(xg).reshape(-1, C), xo.reshape(-1, C), "f32")
    assert not np.allclose(xo, lat.numpy())           # the loop moved the latent
