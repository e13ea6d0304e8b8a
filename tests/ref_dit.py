"""An ordinary full-sequence DiT step written with torch library routines in float64.

Used only to pin the oracle: one block spanning the whole video with an empty
cache must reduce to this.  It is written independently of the oracle: LayerNorm,
softmax attention, GELU and SiLU are torch.nn.functional routines, linear maps
are torch matmuls and the rotary embedding is a complex multiplication.
"""
import math

import torch
import torch.nn.functional as F

T64 = torch.float64


def rope_complex(x, n_heads, head_dim, n_frames, frame0, tok_h, tok_w, theta):
    """x [S, D] -> rotated; each channel pair is a complex number multiplied by exp(i * angle)."""
    S = x.shape[0]
    half = head_dim // 2
    c_sp = head_dim // 6
    c_f = half - 2 * c_sp
    f = (torch.arange(n_frames, dtype=T64) + frame0).view(-1, 1, 1).expand(n_frames, tok_h, tok_w).reshape(-1)
    y = torch.arange(tok_h, dtype=T64).view(1, -1, 1).expand(n_frames, tok_h, tok_w).reshape(-1)
    w = torch.arange(tok_w, dtype=T64).view(1, 1, -1).expand(n_frames, tok_h, tok_w).reshape(-1)

    def freqs(c):
        return theta ** (-torch.arange(c, dtype=T64) / c)

    ang = torch.cat([f[:, None] * freqs(c_f)[None], y[:, None] * freqs(c_sp)[None], w[:, None] * freqs(c_sp)[None]], 1)
    rot = torch.polar(torch.ones_like(ang), ang)                       # [S, half]
    xc = torch.view_as_complex(x.reshape(S, n_heads, half, 2).contiguous())
    return torch.view_as_real(xc * rot[:, None, :]).reshape(S, n_heads * head_dim)


def rms(x, g, eps):
    return x * torch.rsqrt(x.pow(2).mean(-1, keepdim=True) + eps) * g


def mha(q, k, v, n_heads):
    S, D = q.shape
    d = D // n_heads
    qh, kh, vh = (t.reshape(t.shape[0], n_heads, d).transpose(0, 1) for t in (q, k, v))
    o = F.scaled_dot_product_attention(qh, kh, vh)
    return o.transpose(0, 1).reshape(S, D)


def modulation(cfg, ws, t):
    half = cfg["freq_dim"] // 2
    w = torch.exp(-math.log(10000.0) * torch.arange(half, dtype=T64) / half)
    tau = torch.cat([torch.cos(t * w), torch.sin(t * w)])
    e = F.silu(tau @ ws["wt1"] + ws["bt1"]) @ ws["wt2"] + ws["bt2"]
    return (F.silu(e) @ ws["wm"] + ws["bm"]).reshape(6, cfg["dim"])


def text_context(cfg, ws, text):
    if cfg["text_dim"] == cfg["dim"]:
        return text
    return F.gelu(text @ ws["wx1"] + ws["bx1"], approximate="tanh") @ ws["wx2"] + ws["bx2"]


def dit_layer(cfg, lw, x, e0, ctx, n_frames, frame0, extra_kv=None):
    """One DiT layer over the full token sequence x [S, D].  extra_kv: optional (K, V) rows prepended to
    the self-attention keys/values.  Returns (x_out, k_hat, v, attn)."""
    D, h, d, eps = cfg["dim"], cfg["n_heads"], cfg["head_dim"], cfg["eps"]
    sh1, sc1, g1, sh2, sc2, g2 = (lw["mod"] + e0)
    hn = F.layer_norm(x, (D,), eps=eps) * (1 + sc1) + sh1
    geo = (h, d, n_frames, frame0, cfg["tok_h"], cfg["tok_w"], cfg["rope_theta"])
    q = rope_complex(rms(hn @ lw["wq"] + lw["bq"], lw["gq"], eps), *geo)
    k = rope_complex(rms(hn @ lw["wk"] + lw["bk"], lw["gk"], eps), *geo)
    v = hn @ lw["wv"] + lw["bv"]
    ka, va = (k, v) if extra_kv is None else (torch.cat([extra_kv[0], k]), torch.cat([extra_kv[1], v]))
    attn = mha(q, ka, va, h)
    x = x + g1 * (attn @ lw["wo"] + lw["bo"])
    u = F.layer_norm(x, (D,), lw["ln3_g"], lw["ln3_b"], eps)
    cq = rms(u @ lw["cwq"] + lw["cbq"], lw["cgq"], eps)
    ck = rms(ctx @ lw["cwk"] + lw["cbk"], lw["cgk"], eps)
    cv = ctx @ lw["cwv"] + lw["cbv"]
    x = x + mha(cq, ck, cv, h) @ lw["cwo"] + lw["cbo"]
    f_in = F.layer_norm(x, (D,), eps=eps) * (1 + sc2) + sh2
    x = x + g2 * (F.gelu(f_in @ lw["w1"] + lw["b1"], approximate="tanh") @ lw["w2"] + lw["b2"])
    return x, k, v, attn


def full_sequence_step(cfg, weights, text, x, n_frames, frame0, t):
    ws = {k: v.to(T64) for k, v in weights["stage"].items()}
    e0 = modulation(cfg, ws, torch.tensor(float(t), dtype=T64))
    ctx = text_context(cfg, ws, text.to(T64))
    x = x.to(T64)
    for lw in weights["layers"]:
        lw = {k: v.to(T64) for k, v in lw.items()}
        x, _, _, _ = dit_layer(cfg, lw, x, e0, ctx, n_frames, frame0)
    return x
