"""GPU parity at the sizes and in the launch configurations the benchmark times that the other files do
not reach: the Wan-14B-shaped stage at its full 4 + 2 frames (14400-token block, 7200 cached tokens), the
longer first block of the long-video configuration at Wan-1.3B width (5 frames = 7800 tokens, Sec. 3.3), and
that configuration's whole latent-space loop (257 latent frames = 5 + 63 x 4, pool of 6 noise frames) on a
tiny model, every pass against the oracle."""
import numpy as np
import pytest
import torch

from harness import check, gpu_stage, oracle_stage, to_dev, to_np
from oracle.stage import OracleStage, token_positions
from paper_2505_21070_amd import synth

pytestmark = pytest.mark.gpu


def edge_rows(n, step, extra, rng):
    """Row indices that touch every `step`-row tile's first and last row, the very last rows, plus `extra`
    random ones."""
    fixed = [r for t in range(0, n, step) for r in (t, min(t + step - 1, n - 1))] + [n - 1, n - 2]
    return np.unique(np.concatenate([np.array(fixed), rng.choice(n, size=extra, replace=False)]))


def test_wan14b_stage_full_size_teacher_forced(progress):
    """One Wan-14B-shaped layer (dim 5120, 40 heads x 128, FFN 13824, 45 x 80 tokens per frame, 512 text tokens
    of width 4096) at the benchmark's size: a 4-frame block of 14400 tokens attending over itself and the 7200
    cached tokens of the neighbour's first 2 frames.  Keys/values for all 21600 tokens would take the CPU
    oracle minutes, so they are teacher-forced: the oracle computes K-hat and V for ~700 sampled tokens of the
    block and ~500 of the cache (every 256-row tile's first and last row among them) and these are compared
    with the library's; the oracle's attention for 48 sampled query rows then runs over all 21600 keys, taking
    the library's (sample-checked) K-hat / V for the tokens it did not compute itself."""
    cfg, w, text, blocks = synth.make_case("wan14b_stage", seed=1, strong_gate=True, n_layers=1)
    nf, nc, th, tw = cfg["block_frames"], cfg["cache_frames"], cfg["tok_h"], cfg["tok_w"]
    tok = th * tw
    S, Nc = nf * tok, nc * tok
    assert (S, Nc, cfg["dim"]) == (14400, 7200, 5120)
    rng = np.random.default_rng(14)
    progress("inputs drawn; building the stage")
    g = gpu_stage(cfg, w, text, max_abs_frames=8)
    x_nb, x_cur = to_dev(blocks[0], cfg), to_dev(blocks[1], cfg)
    g.forward(x_nb, nf, nf, 625.0)
    g.cache_update(0, nc)
    ck, cv = to_np(g.peek("cache_k", 0)), to_np(g.peek("cache_v", 0))
    assert ck.shape == (Nc, cfg["dim"])
    y = g.forward(x_cur, nf, 0, 500.0)
    torch.cuda.synchronize()
    gk, gv = to_np(g.peek("k", 0)), to_np(g.peek("v", 0))
    xres = to_np(g.peek("x_res", 0))
    progress("GPU done; building the oracle")
    o = OracleStage(cfg, synth.to_numpy(w), text.numpy())
    # cached keys/values: frames [nf, nf + nc) of the neighbour, sampled tokens
    rows_c = edge_rows(Nc, 256, 384, rng)
    pos_nb = token_positions(nc, nf, th, tw)
    _, k_c, v_c = o.layer(0, blocks[0].numpy()[rows_c], o.modulation(625.0), tuple(p[rows_c] for p in pos_nb), None,
                          rows=np.array([0]))
    check("14b/cache_k", ck[rows_c], k_c, "bf16")
    check("14b/cache_v", cv[rows_c], v_c, "bf16")
    progress(f"cache checked on {rows_c.size} rows")
    # the block: sampled tokens (queries among them) computed by the oracle, the rest of the keys teacher-forced
    rows_q = np.unique(np.concatenate([[0, 1, S - 1, tok - 1, tok, 2 * tok, 14336, 14399], rng.choice(S, size=40, replace=False)]))
    rows_s = np.unique(np.concatenate([rows_q, edge_rows(S, 256, 512, rng)]))
    others = np.setdiff1d(np.arange(S), rows_s)
    pos = token_positions(nf, 0, th, tw)
    xin = blocks[1].numpy().astype(np.float64)
    ref, k_s, v_s = o.layer(0, xin[rows_s], o.modulation(500.0), tuple(p[rows_s] for p in pos), (ck, cv),
                            rows=np.searchsorted(rows_s, rows_q), block_kv=(gk[others], gv[others]))
    check("14b/k", gk[rows_s], k_s, "bf16")
    check("14b/v", gv[rows_s], v_s, "bf16")
    rep = {}
    check("14b/x_res", xres[rows_q], ref, "bf16", rep)
    check("14b/delta", xres[rows_q] - xin[rows_q], ref - xin[rows_q], "bf16", rep)
    check("14b/x_out", to_np(y)[rows_q], ref, "bf16", rep)
    progress(str({k: f"{v['rel_l2']:.2e} (worst row {v['worst_row']:.2e})" for k, v in rep.items()}))
    assert torch.isfinite(y.float()).all()


def test_long_video_first_block_at_wan1p3b_width():
    """The long-video configuration's first block (Sec. 3.3: the first block is longer; 257 latent frames =
    5 + 63 x 4) at Wan-1.3B width: 5 frames = 7800 tokens at frames 0..4, attending over the cached first 2
    frames (3120 tokens) of block 2, which sits at frames 5..8 and was processed just before it.  One layer,
    keys/values compared on all rows, the layer output on sampled query rows over all 10920 keys."""
    cfg, w, text, _ = synth.make_case("wan1p3b_stage", seed=4, strong_gate=True, n_blocks=0, n_layers=1)
    th, tw, nc = cfg["tok_h"], cfg["tok_w"], cfg["cache_frames"]
    tok = th * tw
    first, num_b = 5, 4
    gen = torch.Generator().manual_seed(41)
    x2, x1 = synth.make_block(cfg, num_b, gen), synth.make_block(cfg, first, gen)
    g = gpu_stage(cfg, w, text, max_block_frames=first, max_abs_frames=16)
    o = OracleStage(cfg, synth.to_numpy(w), text.numpy())
    g.forward(to_dev(x2, cfg), num_b, first, 1000.0)
    g.cache_update(0, nc)
    _, k_c, v_c = o.layer(0, x2.numpy()[: nc * tok], o.modulation(1000.0), token_positions(nc, first, th, tw), None,
                          rows=np.array([0]))
    check("first/cache_k", to_np(g.peek("cache_k", 0)), k_c, "bf16")
    check("first/cache_v", to_np(g.peek("cache_v", 0)), v_c, "bf16")
    y = g.forward(to_dev(x1, cfg), first, 0, 980.0)
    S = first * tok
    rows = np.unique(np.concatenate([[0, 1, S - 1, S - 2, tok - 1, tok, 4 * tok, 7679, 7680, 7799],
                                     np.random.default_rng(5).choice(S, size=118, replace=False)]))
    xin = x1.numpy().astype(np.float64)
    ref, k, v = o.layer(0, xin, o.modulation(980.0), token_positions(first, 0, th, tw), (k_c, v_c), rows=rows)
    check("first/k", to_np(g.peek("k", 0)), k, "bf16")
    check("first/v", to_np(g.peek("v", 0)), v, "bf16")
    xres = to_np(g.peek("x_res", 0))[rows]
    check("first/x_res", xres, ref, "bf16")
    check("first/delta", xres - xin[rows], ref - xin[rows], "bf16")
    check("first/x_out", to_np(y)[rows], ref, "bf16")
    assert torch.isfinite(y.float()).all()


@pytest.mark.parametrize("name", ["tiny", "tiny_bf16"])
def test_long_video_latent_loop_matches_oracle(name, progress):
    """The long-video configuration end to end on a tiny model: 257 latent frames as one 5-frame block + 63
    blocks of 4, every block's initial noise gathered from the shared pool of 6 frames (Sec. 3.3), T = 3 noise
    levels, the whole queue from the first push to the last pop (192 passes, tail to head, Sec. 3.1).  A pass is
    patch embedding -> stage with the neighbour's cached K/V (Sec. 3.2) -> cache hand-over -> output head ->
    Euler update of the block's latent frames.  Both sides run freely (nothing is teacher-forced); the stage
    output and the updated latent of every pass are compared with the oracle's."""
    from oracle.ends import OracleEnds, euler_step
    from oracle.noise import gather_frames, noise_assignment
    from oracle.schedule import blockwise_schedule as oracle_schedule
    from paper_2505_21070_amd import binding as B
    cfg, w, text, _ = synth.make_case(name, seed=17, strong_gate=True, n_blocks=0, block_frames=4, cache_frames=2)
    dt = cfg["dtype"]
    C, frames, num_b, half, first, block_num, T = 16, 257, 4, 2, 5, 64, 3
    tok = cfg["tok_h"] * cfg["tok_w"]
    td = torch.bfloat16 if dt == "bf16" else torch.float32
    ew = synth.make_end_weights(cfg, C, 17)
    host = {k: v.numpy() for k, v in ew.items()}
    host.update({k: w["stage"][k].numpy() for k in ("wt1", "bt1", "wt2", "bt2")})
    g_ends = B.Ends(cfg, {k: torch.from_numpy(v).to("cuda", td).contiguous() for k, v in host.items()}, C, first)
    o_ends = OracleEnds(dict(cfg, channels=C), host)
    g = gpu_stage(cfg, w, text, max_block_frames=first, max_cache_frames=half, max_abs_frames=frames)
    o = oracle_stage(cfg, w, text)
    # coordinated noise initialisation; block 1 is one frame shorter than the pool here, so it takes the pool's
    # last 5 frames (both sides from the oracle's own assignment, which the library's must equal)
    pool = synth.make_latent(cfg, num_b + half, C, torch.Generator().manual_seed(18))
    words = synth.shuffle_words((block_num - 1) * (num_b - 1), 19)
    idx = noise_assignment(block_num, num_b, 2 * half, words)
    assert B.noise_assign(block_num, num_b, 2 * half, words) == idx
    idx[0] = idx[0][-first:]
    flat = [i for blk in idx for i in blk]
    assert len(flat) == frames
    lat_g = B.noise_gather(pool.cuda(), torch.tensor(flat, dtype=torch.int32, device="cuda"))
    lat_o = gather_frames(pool.numpy().astype(np.float64), flat)
    assert np.array_equal(lat_g.cpu().numpy(), lat_o.astype(np.float32))
    sched = B.blockwise_schedule(T, block_num, num_b, 2 * half, first, 1000.0, "reverse")
    ref_sched = oracle_schedule(T, block_num, num_b, 2 * half, first, 1000.0, "reverse")
    assert len(sched) == T * block_num == len(ref_sched)
    assert max(e["frame0"] + e["n_frames"] for e in sched) == frames
    worst = 0.0
    for p, (e, r) in enumerate(zip(sched, ref_sched)):
        assert all(e[k] == r[k] for k in ("step", "block", "level", "frame0", "n_frames", "cache_block"))
        n, f0, k = e["n_frames"], e["frame0"], e["level"]
        if e["cache_block"] == 0:
            g.cache_update(0, 0); o.cache_update(0, 0)
        yg = g.forward(g_ends.embed(lat_g[f0:f0 + n]), n, f0, e["timestep"])
        yo = o.forward(o_ends.embed(lat_o[f0:f0 + n]), n, f0, r["timestep"])
        g.cache_update(0, half); o.cache_update(0, half)
        rep = {}
        check(f"loop/pass{p}/block{e['block']}/level{k}/y", to_np(yg), yo, dt, rep)
        B.euler_step(lat_g[f0:f0 + n], g_ends.head(yg, e["timestep"], n), k / T, (k - 1) / T)
        lat_o[f0:f0 + n] = euler_step(lat_o[f0:f0 + n], o_ends.head(yo, r["timestep"], n), k / T, (k - 1) / T)
        check(f"loop/pass{p}/block{e['block']}/level{k}/latent", to_np(lat_g[f0:f0 + n]).reshape(n * tok, -1),
              lat_o[f0:f0 + n].reshape(n * tok, -1), dt, rep)
        worst = max(worst, max(v["max_abs"] if dt == "f32" else v["rel_l2"] for v in rep.values()))
        if p % 48 == 47:
            progress(f"{p + 1} of {len(sched)} passes, worst {'max_abs' if dt == 'f32' else 'rel_l2'} so far {worst:.3e}")
    check("loop/final_latent", to_np(lat_g).reshape(frames * tok, -1), lat_o.reshape(frames * tok, -1), dt)
    assert not np.allclose(lat_o, gather_frames(pool.numpy().astype(np.float64), flat))
