"""Seeded synthetic inputs for the block-wise denoising stage.

Holds no arithmetic of the method: only shapes, the random draws and the
rounding of the drawn values to the storage type.  Both the GPU tests/bench
and the CPU oracle's tests take their inputs from here, so the two sides see
the same host arrays.  Random-init weights and N(0,1) latents/text stand in
for trained Wan2.1 weights, VAE latents and T5 text embeddings.

Draw order (one torch CPU generator seeded with `seed`): stage-level weights in
STAGE_ORDER, then for each layer the tensors in LAYER_ORDER, then the text
tensor, then any activations requested, each as fp32 normal draws.
"""
from collections import OrderedDict

import numpy as np
import torch

# name -> stage geometry.  block_frames / cache_frames are the workload's block and cache sizes.
CONFIGS = {
    # 2 layers, dim 128, 2 heads x 64, FFN 512, 2 frames x 8x8 tokens + 1 cached frame, 16 text tokens
    "tiny": dict(n_layers=2, dim=128, n_heads=2, head_dim=64, ffn_dim=512, text_len=16, text_dim=128,
                 tok_h=8, tok_w=8, block_frames=2, cache_frames=1, dtype="f32"),
    # same geometry at bf16 storage, for whole-stage bf16 parity against the full oracle
    "tiny_bf16": dict(n_layers=2, dim=128, n_heads=2, head_dim=64, ffn_dim=512, text_len=16, text_dim=128,
                      tok_h=8, tok_w=8, block_frames=2, cache_frames=1, dtype="bf16"),
    # a small ragged bf16 case: head_dim 128, token counts that are not tile multiples, text MLP present
    "small_bf16": dict(n_layers=2, dim=256, n_heads=2, head_dim=128, ffn_dim=640, text_len=40, text_dim=192,
                       tok_h=6, tok_w=12, block_frames=3, cache_frames=2, dtype="bf16"),
    # the same ragged shape in fp32, with odd token and text counts (7 x 9 tokens per frame, 37 text tokens)
    "small_f32": dict(n_layers=2, dim=256, n_heads=2, head_dim=128, ffn_dim=640, text_len=37, text_dim=192,
                      tok_h=7, tok_w=9, block_frames=3, cache_frames=2, dtype="f32"),
    # few queries against a long ragged key range (31.5 key tiles): the attention grid is small enough
    # that its work is cut into key ranges which a second kernel merges
    "longkv_bf16": dict(n_layers=1, dim=128, n_heads=2, head_dim=64, ffn_dim=256, text_len=24, text_dim=128,
                        tok_h=16, tok_w=21, block_frames=3, cache_frames=3, dtype="bf16"),
    # enough (head, 256-query block) pairs and keys for the attention kernel's 256-query block shape at
    # head_dim 64, with its work ids cut into two key ranges
    "wide64_bf16": dict(n_layers=1, dim=1024, n_heads=16, head_dim=64, ffn_dim=1024, text_len=32, text_dim=1024,
                        tok_h=16, tok_w=16, block_frames=8, cache_frames=2, dtype="bf16"),
    # head_dim 128 with enough rows and columns for the GEMM's 256 x 256 tiles (72 of them in the fused
    # q|k|v projection, whose epilogue writes per head) and the attention kernel's 256-query blocks
    "wide128_bf16": dict(n_layers=1, dim=768, n_heads=6, head_dim=128, ffn_dim=1024, text_len=48, text_dim=768,
                         tok_h=16, tok_w=16, block_frames=8, cache_frames=2, dtype="bf16"),
    # dim % 256 != 0, so q|k|v and the cross-attention query take the plain store epilogue and the separate
    # norm / rotation / transpose kernels, at row counts that make the GEMM choose its other tile shapes for
    # every epilogue: 4032 rows -> 192 x 256 tiles, 4096 rows -> 256 x 256, 4160 rows with dim 1408 -> 320 x 256
    # (q|k|v) and 160 x 256 (the rest)
    "tile192_bf16": dict(n_layers=1, dim=896, n_heads=7, head_dim=128, ffn_dim=1024, text_len=40, text_dim=896,
                         tok_h=14, tok_w=36, block_frames=8, cache_frames=2, dtype="bf16"),
    "tile256_bf16": dict(n_layers=1, dim=896, n_heads=7, head_dim=128, ffn_dim=1024, text_len=40, text_dim=896,
                         tok_h=16, tok_w=32, block_frames=8, cache_frames=2, dtype="bf16"),
    "tile320_bf16": dict(n_layers=1, dim=1408, n_heads=11, head_dim=128, ffn_dim=1024, text_len=40, text_dim=1408,
                         tok_h=20, tok_w=26, block_frames=8, cache_frames=2, dtype="bf16"),
    # few tokens, wide models: the widest register variants of the row kernels (LayerNorm, deferred key scale,
    # norm + rotation); 6144 takes the per-head GEMM epilogue, 2176 = 17 x 128 the separate kernels
    "dim6144_bf16": dict(n_layers=1, dim=6144, n_heads=48, head_dim=128, ffn_dim=512, text_len=24, text_dim=6144,
                         tok_h=8, tok_w=8, block_frames=2, cache_frames=1, dtype="bf16"),
    "dim2176_bf16": dict(n_layers=1, dim=2176, n_heads=17, head_dim=128, ffn_dim=640, text_len=24, text_dim=2176,
                         tok_h=8, tok_w=8, block_frames=2, cache_frames=1, dtype="bf16"),
    # Wan-1.3B-shaped stage: 4 of 30 layers, 4 frames x 30x52 tokens + 2 cached frames
    "wan1p3b_stage": dict(n_layers=4, dim=1536, n_heads=12, head_dim=128, ffn_dim=8960, text_len=512,
                          text_dim=4096, tok_h=30, tok_w=52, block_frames=4, cache_frames=2, dtype="bf16"),
    # all 30 layers on one GPU (block queue workloads)
    "wan1p3b_full": dict(n_layers=30, dim=1536, n_heads=12, head_dim=128, ffn_dim=8960, text_len=512,
                         text_dim=4096, tok_h=30, tok_w=52, block_frames=4, cache_frames=2, dtype="bf16"),
    # Wan-14B-shaped stage: 5 of 40 layers, 4 frames x 45x80 tokens + 2 cached frames
    "wan14b_stage": dict(n_layers=5, dim=5120, n_heads=40, head_dim=128, ffn_dim=13824, text_len=512,
                         text_dim=4096, tok_h=45, tok_w=80, block_frames=4, cache_frames=2, dtype="bf16"),
}
DEFAULTS = dict(freq_dim=256, rope_theta=1.0e4, eps=1.0e-6)

STAGE_ORDER = ("wt1", "bt1", "wt2", "bt2", "wm", "bm", "wx1", "bx1", "wx2", "bx2")
LAYER_ORDER = ("mod", "wq", "bq", "wk", "bk", "wv", "bv", "gq", "gk", "wo", "bo", "ln3_g", "ln3_b",
               "cwq", "cbq", "cgq", "cwk", "cbk", "cgk", "cwv", "cbv", "cwo", "cbo", "w1", "b1", "w2", "b2")
GAINS = ("gq", "gk", "ln3_g", "cgq", "cgk")        # drawn as 1 + 0.02 N(0,1)


def stage_config(name, **over):
    cfg = dict(CONFIGS[name])
    cfg.update(DEFAULTS)
    cfg.update(over)
    return cfg


def weight_shapes(cfg):
    D, F, Td, fd = cfg["dim"], cfg["ffn_dim"], cfg["text_dim"], cfg["freq_dim"]
    stage = OrderedDict(wt1=(fd, D), bt1=(D,), wt2=(D, D), bt2=(D,), wm=(D, 6 * D), bm=(6 * D,))
    if Td != D:
        stage.update(wx1=(Td, D), bx1=(D,), wx2=(D, D), bx2=(D,))
    layer = OrderedDict()
    for k in LAYER_ORDER:
        if k == "mod":
            layer[k] = (6, D)
        elif k == "w1":
            layer[k] = (D, F)
        elif k == "b1":
            layer[k] = (F,)
        elif k == "w2":
            layer[k] = (F, D)
        elif k.startswith("w") or k.startswith("cw"):
            layer[k] = (D, D)
        else:
            layer[k] = (D,)
    return stage, layer


def round_to(t, dtype):
    """fp32 tensor holding values representable in the storage type (round-to-nearest-even)."""
    if dtype == "bf16":
        return t.to(torch.bfloat16).to(torch.float32)
    return t


def make_weights(cfg, seed=0, strong_gate=False, gen=None):
    """{"stage": {name: fp32 tensor}, "layers": [{name: fp32 tensor}]}, values already rounded to
    cfg["dtype"].  Matrices are [in, out] row-major.  strong_gate: the three gate rows of each layer's
    modulation table are drawn around 1 instead of 0 so that branch outputs are not scaled away."""
    g = gen if gen is not None else torch.Generator(device="cpu").manual_seed(seed)
    sshape, lshape = weight_shapes(cfg)

    def draw(shape, mean=0.0):
        return mean + 0.02 * torch.randn(shape, generator=g, dtype=torch.float32)

    stage = OrderedDict((k, round_to(draw(s), cfg["dtype"])) for k, s in sshape.items())
    layers = []
    for _ in range(cfg["n_layers"]):
        lw = OrderedDict()
        for k, s in lshape.items():
            t = draw(s, 1.0 if k in GAINS else 0.0)
            if k == "mod" and strong_gate:
                t[2] += 1.0
                t[5] += 1.0
            lw[k] = round_to(t, cfg["dtype"])
        layers.append(lw)
    return {"stage": stage, "layers": layers}


def make_text(cfg, gen):
    return round_to(torch.randn((cfg["text_len"], cfg["text_dim"]), generator=gen, dtype=torch.float32), cfg["dtype"])


def make_block(cfg, n_frames, gen):
    """N(0,1) hidden tokens of one block: [n_frames * tok_h * tok_w, dim]."""
    S = n_frames * cfg["tok_h"] * cfg["tok_w"]
    return round_to(torch.randn((S, cfg["dim"]), generator=gen, dtype=torch.float32), cfg["dtype"])


def make_case(name, seed=0, strong_gate=False, n_blocks=2, **over):
    """Config, weights, text and `n_blocks` blocks of cfg["block_frames"] frames, all from one seed."""
    cfg = stage_config(name, **over)
    g = torch.Generator(device="cpu").manual_seed(seed)
    weights = make_weights(cfg, strong_gate=strong_gate, gen=g)
    text = make_text(cfg, g)
    blocks = [make_block(cfg, cfg["block_frames"], g) for _ in range(n_blocks)]
    return cfg, weights, text, blocks


def to_numpy(weights):
    return {"stage": {k: v.numpy() for k, v in weights["stage"].items()},
            "layers": [{k: v.numpy() for k, v in lw.items()} for lw in weights["layers"]]}


def shuffle_words(n, seed):
    """n unsigned 32-bit random words (the random numbers the noise initialisation consumes), from one seed."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    return [int(v) for v in torch.randint(0, 2**32, (n,), generator=g, dtype=torch.int64)]


def noise_pool(cfg, pool_frames, gen):
    """Token-space stand-in for the shared initial-noise pool: [pool_frames, tokens per frame, dim] N(0,1)."""
    tok = cfg["tok_h"] * cfg["tok_w"]
    return round_to(torch.randn((pool_frames, tok, cfg["dim"]), generator=gen, dtype=torch.float32), cfg["dtype"])


def make_end_weights(cfg, channels=16, seed=0):
    """Weights of the model's two ends (patch embedding, output head), N(0, 0.02) like the rest, rounded to
    cfg["dtype"]; matrices [in, out].  Keys: w_pe [4C, dim], b_pe, m_head [2, dim], w_head [dim, 4C], b_head."""
    g = torch.Generator(device="cpu").manual_seed(seed + 7777)
    D, P = cfg["dim"], 4 * channels
    shapes = OrderedDict(w_pe=(P, D), b_pe=(D,), m_head=(2, D), w_head=(D, P), b_head=(P,))
    return OrderedDict((k, round_to(0.02 * torch.randn(sh, generator=g, dtype=torch.float32), cfg["dtype"]))
                       for k, sh in shapes.items())


def make_latent(cfg, n_frames, channels, gen):
    """N(0,1) frame latents [n_frames, 2*tok_h, 2*tok_w, channels], fp32 (latents are kept in fp32)."""
    return torch.randn((n_frames, 2 * cfg["tok_h"], 2 * cfg["tok_w"], channels), generator=gen, dtype=torch.float32)
