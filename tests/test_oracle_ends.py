"""Pins of the oracle's model ends (patch embedding, output head) and scheduler step."""
import numpy as np
import pytest
import torch

from oracle.ends import OracleEnds, euler_step, patchify, unpatchify
from oracle.stage import OracleStage
from paper_2505_21070_amd import synth


def _ends(name="tiny", channels=4, seed=0):
    cfg = synth.stage_config(name)
    w = synth.make_weights(cfg, seed=seed)
    ew = synth.make_end_weights(cfg, channels, seed)
    weights = {k: v.numpy() for k, v in ew.items()}
    weights.update({k: w["stage"][k].numpy() for k in ("wt1", "bt1", "wt2", "bt2")})
    return cfg, w, OracleEnds(dict(cfg, channels=channels), weights)


def test_patchify_layout_and_inverse():
    F, H, W, C = 2, 4, 6, 3
    lat = np.arange(F * H * W * C, dtype=np.float64).reshape(F, H, W, C)
    tok = patchify(lat)
    assert tok.shape == (F * 2 * 3, 4 * C)
    # token (f=1, y=1, x=2), value (dy=1, dx=0, c=2) is pixel (1, 3, 4, 2); brute force over everything
    assert tok[1 * 6 + 1 * 3 + 2, (1 * 2 + 0) * C + 2] == lat[1, 3, 4, 2]
    for f in range(F):
        for y in range(H // 2):
            for x in range(W // 2):
                for dy in range(2):
                    for dx in range(2):
                        for c in range(C):
                            assert tok[(f * 2 + y) * 3 + x, (dy * 2 + dx) * C + c] == lat[f, 2 * y + dy, 2 * x + dx, c]
    assert np.array_equal(unpatchify(tok, F, H, W, C), lat)
    assert np.array_equal(patchify(unpatchify(tok, F, H, W, C)), tok)


def test_embed_is_a_strided_convolution():
    cfg, _, ends = _ends()
    C = 4
    gen = torch.Generator().manual_seed(1)
    lat = synth.make_latent(cfg, 2, C, gen).numpy().astype(np.float64)
    got = ends.embed(lat)
    # the same thing as a 1x2x2 convolution with stride (1,2,2), via torch, weight [D, C, 1, 2, 2]
    w = np.asarray(ends.w["w_pe"]).reshape(2, 2, C, cfg["dim"])                    # (dy, dx, c, out)
    wt = torch.from_numpy(np.ascontiguousarray(w.transpose(3, 2, 0, 1)))[:, :, None]   # [out, c, 1, dy, dx]
    x = torch.from_numpy(lat).permute(3, 0, 1, 2)[None]                             # [1, C, F, H, W]
    ref = torch.nn.functional.conv3d(x, wt, torch.from_numpy(np.asarray(ends.w["b_pe"])), stride=(1, 2, 2))
    ref = ref[0].permute(1, 2, 3, 0).reshape(-1, cfg["dim"]).numpy()
    assert np.allclose(got, ref, rtol=0, atol=1e-12)


def test_head_against_library_routines_and_shares_the_stage_time_embedding():
    cfg, w, ends = _ends(seed=3)
    C = 4
    gen = torch.Generator().manual_seed(2)
    S = 2 * cfg["tok_h"] * cfg["tok_w"]
    x = torch.randn((S, cfg["dim"]), generator=gen, dtype=torch.float64)
    got = ends.head(x.numpy(), 437.0, 2)
    assert got.shape == (2, 2 * cfg["tok_h"], 2 * cfg["tok_w"], C)
    e = torch.from_numpy(np.asarray(ends.time_embedding(437.0)))
    mh = torch.from_numpy(np.asarray(ends.w["m_head"]))
    y = torch.nn.functional.layer_norm(x, (cfg["dim"],), eps=cfg["eps"]) * (1 + mh[1] + e) + (mh[0] + e)
    out = y @ torch.from_numpy(np.asarray(ends.w["w_head"])) + torch.from_numpy(np.asarray(ends.w["b_head"]))
    assert np.allclose(got, unpatchify(out.numpy(), 2, 2 * cfg["tok_h"], 2 * cfg["tok_w"], C), rtol=0, atol=1e-12)
    # the head's timestep embedding is the vector the stage projects to its 6*dim modulation
    st = OracleStage(cfg, synth.to_numpy(w), synth.make_text(cfg, gen).numpy())
    e0 = st.ops.linear(st.ops.silu(np.asarray(e)[None, :]), st.w["wm"], st.w["bm"]).reshape(6, cfg["dim"])
    assert np.allclose(e0, st.modulation(437.0), rtol=0, atol=1e-13)
    # scale and shift are not interchanged: zero weights leave the bias, a zero input leaves shift W + b
    z = ends.head(np.zeros((S, cfg["dim"])), 437.0, 2)
    shift = (mh[0] + e) @ torch.from_numpy(np.asarray(ends.w["w_head"])) + torch.from_numpy(np.asarray(ends.w["b_head"]))
    assert np.allclose(patchify(z)[5], shift.numpy(), atol=1e-12)


def test_euler_step_closed_forms():
    rng = np.random.default_rng(0)
    x1, x0 = rng.standard_normal((3, 4, 4, 2)), rng.standard_normal((3, 4, 4, 2))
    # straight path x_sigma = (1 - sigma) x0 + sigma x1 has constant velocity x1 - x0: T equal steps from
    # sigma = 1 land on x0, whatever T
    for T in (1, 4, 50):
        x = x1.copy()
        for k in range(T, 0, -1):
            x = euler_step(x, x1 - x0, k / T, (k - 1) / T)
        assert np.allclose(x, x0, atol=1e-12)
    # one step is linear in v and moves against v when sigma decreases
    v = rng.standard_normal(x1.shape)
    assert np.allclose(euler_step(x1, v, 0.5, 0.25), x1 - 0.25 * v)
    assert np.array_equal(euler_step(x1, v, 0.3, 0.3), x1)
