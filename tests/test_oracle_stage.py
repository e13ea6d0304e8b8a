"""Pins of the oracle's stage: the properties that fix cache wiring, RoPE offsets, modulation and
layer order independently of the oracle's own code."""
import numpy as np
import pytest
import torch

import ref_dit
from oracle.stage import OracleStage, token_positions
from paper_2505_21070_amd import synth

T64 = torch.float64


def make(name="tiny", seed=0, strong_gate=True, **over):
    cfg, w, text, blocks = synth.make_case(name, seed=seed, strong_gate=strong_gate, **over)
    return cfg, w, text, blocks, OracleStage(cfg, synth.to_numpy(w), text.numpy())


@pytest.mark.parametrize("name", ["tiny", "small_bf16"])
def test_whole_video_block_is_ordinary_dit_step(oracle_built, name):
    """One block spanning the whole video, empty cache == full-sequence DiT step from library routines."""
    cfg, w, text, blocks, st = make(name)
    nf = cfg["block_frames"]
    got = st.forward(blocks[0].numpy(), nf, 3, 437.0)
    ref = ref_dit.full_sequence_step(cfg, w, text, blocks[0], nf, 3, 437.0).numpy()
    assert np.abs(ref - blocks[0].numpy()).max() > 0.2          # the step does something
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-10)


def test_cached_attention_equals_recompute_over_concatenation(oracle_built):
    """Layer-1 self-attention with the neighbour's cached K/V == attention recomputed from scratch over
    the explicitly concatenated frames (neighbour frames normalised/modulated at the neighbour's noise
    level and rotated at their own absolute frame offsets)."""
    cfg, w, text, blocks, st = make("tiny")
    tok = cfg["tok_h"] * cfg["tok_w"]
    x_nb, x_cur = blocks[0], blocks[1]
    t_nb, t_cur = 625.0, 500.0
    st.forward(x_nb.numpy(), 2, 2, t_nb)          # neighbour block: frames 2..3
    st.cache_update(0, 1)                         # keep its first frame (the one touching frames 0..1)
    taps = []
    st.forward(x_cur.numpy(), 2, 0, t_cur, taps)
    # from scratch, with library routines
    ws = {k: v.to(T64) for k, v in w["stage"].items()}
    lw = {k: v.to(T64) for k, v in w["layers"][0].items()}
    ctx = ref_dit.text_context(cfg, ws, text.to(T64))
    e_nb = ref_dit.modulation(cfg, ws, torch.tensor(t_nb, dtype=T64))
    e_cur = ref_dit.modulation(cfg, ws, torch.tensor(t_cur, dtype=T64))
    _, k_nb, v_nb, _ = ref_dit.dit_layer(cfg, lw, x_nb.to(T64)[:tok], e_nb, ctx, 1, 2)
    # (K/V rows of a frame do not depend on the other frames in layer 1: LN, projections and RoPE are per token)
    _, _, _, attn = ref_dit.dit_layer(cfg, lw, x_cur.to(T64), e_cur, ctx, 2, 0, extra_kv=(k_nb, v_nb))
    np.testing.assert_allclose(taps[0]["attn"], attn.numpy(), rtol=0, atol=1e-11)
    # and the cache changes the result (the test is not vacuous)
    st2 = OracleStage(cfg, synth.to_numpy(w), text.numpy())
    taps2 = []
    st2.forward(x_cur.numpy(), 2, 0, t_cur, taps2)
    assert np.abs(taps2[0]["attn"] - taps[0]["attn"]).max() > 1e-3


def test_empty_cache_and_cleared_cache_agree(oracle_built):
    cfg, w, text, blocks, st = make("tiny")
    a = st.forward(blocks[1].numpy(), 2, 0, 500.0)
    st.cache_update(0, 1)
    b = st.forward(blocks[1].numpy(), 2, 0, 500.0)
    assert np.abs(a - b).max() > 1e-4
    st.cache_update(0, 0)
    np.testing.assert_array_equal(st.forward(blocks[1].numpy(), 2, 0, 500.0), a)


def test_stage_split_chains(oracle_built):
    """Eq. 1: running layers [0,1) then [1,2) as two stages, each with its own cache, equals one stage."""
    cfg, w, text, blocks, st = make("tiny")
    wn = synth.to_numpy(w)
    halves = []
    for li in range(2):
        c = dict(cfg, n_layers=1)
        halves.append(OracleStage(c, {"stage": wn["stage"], "layers": [wn["layers"][li]]}, text.numpy()))
    def run(stages, x, nf, f0, t):
        for s in stages:
            x = s.forward(x, nf, f0, t)
        return x
    run([st], blocks[0].numpy(), 2, 2, 625.0); st.cache_update(0, 1)
    run(halves, blocks[0].numpy(), 2, 2, 625.0); [s.cache_update(0, 1) for s in halves]
    np.testing.assert_allclose(run(halves, blocks[1].numpy(), 2, 0, 500.0),
                               run([st], blocks[1].numpy(), 2, 0, 500.0), rtol=0, atol=1e-12)


def test_common_frame_shift_leaves_outputs_unchanged(oracle_built):
    """Relative-position property: moving the block and its cache source by the same number of frames
    changes nothing."""
    outs = []
    for shift in (0, 37):
        cfg, w, text, blocks, st = make("tiny")
        st.forward(blocks[0].numpy(), 2, 2 + shift, 625.0)
        st.cache_update(0, 1)
        outs.append(st.forward(blocks[1].numpy(), 2, 0 + shift, 500.0))
    np.testing.assert_allclose(outs[0], outs[1], rtol=0, atol=1e-9)
    # moving only the block does change it
    cfg, w, text, blocks, st = make("tiny")
    st.forward(blocks[0].numpy(), 2, 2, 625.0)
    st.cache_update(0, 1)
    assert np.abs(st.forward(blocks[1].numpy(), 2, 5, 500.0) - outs[0]).max() > 1e-4


def test_sampled_rows_match_full_layer(oracle_built):
    cfg, w, text, blocks, st = make("small_bf16")
    nf = cfg["block_frames"]
    x = blocks[0].numpy().astype(np.float64)
    e0 = st.modulation(300.0)
    pos = token_positions(nf, 4, cfg["tok_h"], cfg["tok_w"])
    full, k, v = st.layer(0, x, e0, pos, None)
    rows = np.array([0, 7, 59, 60, 179])
    part, k2, v2 = st.layer(0, x, e0, pos, None, rows=rows)
    np.testing.assert_allclose(part, full[rows], rtol=0, atol=1e-12)
    np.testing.assert_array_equal(k, k2)


def test_teacher_forced_block_keys_match_full_layer(oracle_built):
    """The layer fed only sampled tokens, with the other tokens' keys/values handed in (here: those of the full
    run), gives the full layer's rows: the hook used at sizes where keys/values for every token take minutes."""
    cfg, w, text, blocks, st = make("small_bf16")
    nf, nc = cfg["block_frames"], cfg["cache_frames"]
    tok = cfg["tok_h"] * cfg["tok_w"]
    st.forward(blocks[0].numpy(), nf, nf, 625.0)
    st.cache_update(0, nc)
    cache = st.cache[0]
    x = blocks[1].numpy().astype(np.float64)
    e0 = st.modulation(500.0)
    pos = token_positions(nf, 0, cfg["tok_h"], cfg["tok_w"])
    full, k, v = st.layer(0, x, e0, pos, cache)
    sample = np.array([0, 3, 71, 72, 100, nf * tok - 1])
    others = np.setdiff1d(np.arange(nf * tok), sample)
    q_rows = np.array([1, 4, 5])                       # positions inside `sample`
    part, k_s, v_s = st.layer(0, x[sample], e0, tuple(p[sample] for p in pos), cache, rows=q_rows,
                              block_kv=(k[others], v[others]))
    np.testing.assert_allclose(part, full[sample[q_rows]], rtol=0, atol=1e-12)
    np.testing.assert_array_equal(k_s, k[sample])
    np.testing.assert_array_equal(v_s, v[sample])
    # leaving the other tokens' keys out changes the rows (the hook is not vacuous)
    alone, _, _ = st.layer(0, x[sample], e0, tuple(p[sample] for p in pos), cache, rows=q_rows)
    assert np.abs(alone - part).max() > 1e-4


def test_cache_memory_bound(oracle_built):
    """Live cache per layer is Num_C/2 frames of K and V (appendix efficiency analysis)."""
    cfg, w, text, blocks, st = make("tiny")
    st.forward(blocks[0].numpy(), 2, 2, 625.0)
    st.cache_update(0, 1)
    tok = cfg["tok_h"] * cfg["tok_w"]
    for k, v in st.cache:
        assert k.shape == v.shape == (1 * tok, cfg["dim"])
