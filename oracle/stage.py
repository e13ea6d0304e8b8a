"""Oracle of one pipeline stage of block-wise denoising (TEST INFRASTRUCTURE).

A stage is the model chunk E_theta_j of the paper's device pipeline (Sec. 2,
Eq. 1): a frame block's hidden tokens eps^{j-1} in R^{p x h} go through the
stage's consecutive DiT layers and come out as eps^j.  Each layer keeps the
self-attention key/value features of the block it processed last; the next
block processed (the neighbour at a lower noise level) attends over
[cached K/V ; its own K/V] instead of having the neighbour's frames
concatenated to its input; cross-attention and the FFN only ever see the
current block's tokens (Sec. 3.2).

The paper treats the DiT layer as a black box.  The layer internals below
(adaLN modulation from the timestep, LayerNorm, full-width q/k RMSNorm, 3D
RoPE at absolute frame offsets, cross-attention to text, tanh-GELU FFN) are
the build's stated readings of a Wan-shaped layer; steps are taken one after
another in that order with the plain primitives of `ops`, nothing fused.
"""
import numpy as np

from .ops import Ops

LAYER_KEYS = (
    "mod",                                   # [6, D] learned per-layer modulation table m_l
    "wq", "bq", "wk", "bk", "wv", "bv",      # self-attention projections, [D, D] / [D]
    "gq", "gk",                              # q/k RMSNorm gains [D]
    "wo", "bo",
    "ln3_g", "ln3_b",                        # affine LayerNorm before cross-attention
    "cwq", "cbq", "cgq", "cwk", "cbk", "cgk", "cwv", "cbv", "cwo", "cbo",
    "w1", "b1", "w2", "b2",                  # FFN [D, F], [F], [F, D], [D]
)
STAGE_KEYS = ("wt1", "bt1", "wt2", "bt2", "wm", "bm")   # timestep MLP and 6D modulation head
TEXT_KEYS = ("wx1", "bx1", "wx2", "bx2")                # text MLP (only when text_dim != dim)


def token_positions(n_frames, frame0, tok_h, tok_w):
    """(frame, row, column) of every token of a block; tokens are frame-major, then row-major."""
    f, y, x = np.meshgrid(np.arange(n_frames) + frame0, np.arange(tok_h), np.arange(tok_w), indexing="ij")
    return (f.reshape(-1).astype(np.int32), y.reshape(-1).astype(np.int32), x.reshape(-1).astype(np.int32))


class OracleStage:
    """cfg: dict with n_layers, dim, n_heads, head_dim, ffn_dim, text_len, text_dim, tok_h, tok_w,
    freq_dim, rope_theta, eps.  weights: {"stage": {...}, "layers": [{...}, ...]} of arrays."""

    def __init__(self, cfg, weights, text, real="f64"):
        self.cfg = dict(cfg)
        self.ops = Ops(real)
        a = self.ops.arr
        self.w = {k: a(v) for k, v in weights["stage"].items()}
        self.layers = [{k: a(v) for k, v in lw.items()} for lw in weights["layers"]]
        assert len(self.layers) == cfg["n_layers"]
        assert cfg["n_heads"] * cfg["head_dim"] == cfg["dim"]
        self.tok = cfg["tok_h"] * cfg["tok_w"]
        # text side, once per prompt: optional MLP text_dim -> dim -> dim, then per-layer K_t, V_t
        c = a(text)
        if cfg["text_dim"] != cfg["dim"]:
            c = self.ops.linear(c, self.w["wx1"], self.w["bx1"])
            c = self.ops.gelu_tanh(c)
            c = self.ops.linear(c, self.w["wx2"], self.w["bx2"])
        self.text_ctx = c
        self.text_k, self.text_v = [], []
        for lw in self.layers:
            kt = self.ops.linear(c, lw["cwk"], lw["cbk"])
            self.text_k.append(self.ops.rmsnorm(kt, lw["cgk"], cfg["eps"]))
            self.text_v.append(self.ops.linear(c, lw["cwv"], lw["cbv"]))
        # feature cache: per layer (K, V) of the retained frames of the last block, or None
        self.cache = [None] * cfg["n_layers"]
        self.last_kv = [None] * cfg["n_layers"]     # K-hat, V of the block just processed
        self.last_frames = 0

    # -- adaLN modulation from the timestep --------------------------------
    def modulation(self, t):
        o, w = self.ops, self.w
        tau = o.sinusoid(t, self.cfg["freq_dim"])[None, :]
        e = o.linear(o.silu(o.linear(tau, w["wt1"], w["bt1"])), w["wt2"], w["bt2"])
        e0 = o.linear(o.silu(e), w["wm"], w["bm"])          # [1, 6D]
        return e0.reshape(6, self.cfg["dim"])

    # -- one layer -----------------------------------------------------------
    def layer(self, li, x, e0, pos, cache_kv, taps=None, rows=None, block_kv=None):
        """x: [S, D] layer input for the whole block.  pos: (pf, py, px) of the block's tokens.
        cache_kv: (K_c, V_c) or None.  rows: optional index array; when given only those query rows
        are carried through (keys/values still come from every token) and the result is [len(rows), D].
        block_kv: optional (K-hat, V) of tokens of the block that are NOT among the rows of x, computed
        elsewhere (teacher forcing at sizes where keys/values for every token take minutes of CPU: x then
        holds sampled tokens only, whose own keys/values are computed here and checked by the caller, and
        the given rows are appended to the key/value list; softmax does not care about key order).
        Returns (x_out, K-hat, V) with K-hat, V those computed here from x."""
        o, cfg, lw = self.ops, self.cfg, self.layers[li]
        h, d, eps = cfg["n_heads"], cfg["head_dim"], cfg["eps"]
        sh1, sc1, g1, sh2, sc2, g2 = (lw["mod"] + e0)
        pf, py, px = pos
        # self-attention: keys/values from every token of the block
        hn = o.layernorm(x, eps, 1.0 + sc1, sh1)
        k = o.rope3d(o.rmsnorm(o.linear(hn, lw["wk"], lw["bk"]), lw["gk"], eps), h, d, pf, py, px, cfg["rope_theta"])
        v = o.linear(hn, lw["wv"], lw["bv"])
        if rows is not None:
            x, hn = x[rows], hn[rows]
            pf, py, px = pf[rows], py[rows], px[rows]
        q = o.rope3d(o.rmsnorm(o.linear(hn, lw["wq"], lw["bq"]), lw["gq"], eps), h, d, pf, py, px, cfg["rope_theta"])
        k_all, v_all = k, v
        if cache_kv is not None:
            k_all = np.concatenate([cache_kv[0], k_all], axis=0)
            v_all = np.concatenate([cache_kv[1], v_all], axis=0)
        if block_kv is not None:
            k_all = np.concatenate([k_all, o.arr(block_kv[0])], axis=0)
            v_all = np.concatenate([v_all, o.arr(block_kv[1])], axis=0)
        attn = o.attention(q, k_all, v_all, h)
        x1 = x + g1 * o.linear(attn, lw["wo"], lw["bo"])
        # cross-attention to the text tokens (current block only, no gate, no RoPE)
        u = o.layernorm(x1, eps, lw["ln3_g"], lw["ln3_b"])
        cq = o.rmsnorm(o.linear(u, lw["cwq"], lw["cbq"]), lw["cgq"], eps)
        cattn = o.attention(cq, self.text_k[li], self.text_v[li], h)
        x2 = x1 + o.linear(cattn, lw["cwo"], lw["cbo"])
        # FFN
        f_in = o.layernorm(x2, eps, 1.0 + sc2, sh2)
        mid = o.gelu_tanh(o.linear(f_in, lw["w1"], lw["b1"]))
        y = o.linear(mid, lw["w2"], lw["b2"])
        x3 = x2 + g2 * y
        if taps is not None:
            taps.append({"q": q, "k": k, "v": v, "attn": attn, "x_self": x1, "cattn": cattn,
                         "x_cross": x2, "ffn": y, "x_out": x3})
        return x3, k, v

    # -- the stage -----------------------------------------------------------
    def forward(self, x, n_frames, frame0, t, taps=None):
        """All layers on one block.  Reads each layer's cache, retains the block's K-hat/V."""
        x = self.ops.arr(x)
        assert x.shape == (n_frames * self.tok, self.cfg["dim"])
        e0 = self.modulation(t)
        pos = token_positions(n_frames, frame0, self.cfg["tok_h"], self.cfg["tok_w"])
        for li in range(self.cfg["n_layers"]):
            x, k, v = self.layer(li, x, e0, pos, self.cache[li], taps)
            self.last_kv[li] = (k, v)
        self.last_frames = n_frames
        return x

    def cache_update(self, first_frame, n_frames):
        """Cache <- K-hat, V of frames [first_frame, first_frame + n_frames) of the block processed
        last, in every layer.  n_frames == 0 empties the cache."""
        if n_frames == 0:
            self.cache = [None] * self.cfg["n_layers"]
            return
        assert self.last_frames > 0 and 0 <= first_frame and first_frame + n_frames <= self.last_frames
        a, b = first_frame * self.tok, (first_frame + n_frames) * self.tok
        self.cache = [(k[a:b].copy(), v[a:b].copy()) for (k, v) in self.last_kv]
