"""Oracle of the two ends of the denoising model and of the scheduler update (TEST INFRASTRUCTURE).

The paper (Sec. 2) denoises a frame latent x_t in R^{F x H x W x C}, feeds the model p = F x H' x W' tokens of
hidden size h (H', W' the downsampled H, W), gets the prediction eps_t back in latent shape and updates
x_{t-1} = S(eps_t, x_t, t) with "the updating scheduler of the corresponding video diffusion model".  It
says nothing else about these steps; what follows is this build's stated reading of a Wan-shaped model:

  patch embedding   a token is one 1 x 2 x 2 patch of the latent: (f, y, x) takes pixels (f, 2y+dy, 2x+dx, c)
                    flattened with dy slowest and c fastest (4C values), times W_pe [4C, h] plus b_pe
  output head       e = the timestep embedding (the h-vector before the 6h modulation projection);
                    (shift, scale) = m_head[2, h] + e;  y = LayerNorm(x) * (1 + scale) + shift (no affine);
                    out = y W_head [h, 4C] + b_head, scattered back to the pixels of each token's patch
  scheduler step    flow-matching Euler: the model's output is a velocity v and
                    x <- x + (sigma_next - sigma) v with sigma = t / t_max (level k of T: sigma = k / T)

Each step is taken with the plain primitives of `ops`, in this order, nothing fused.
"""
import numpy as np

from .ops import Ops

END_KEYS = ("w_pe", "b_pe", "m_head", "w_head", "b_head")     # plus the stage's wt1, bt1, wt2, bt2


def patchify(latent):
    """[F, H, W, C] -> [F * H/2 * W/2, 4C]; tokens frame-major then row-major, values ordered (dy, dx, c)."""
    F, H, W, C = latent.shape
    assert H % 2 == 0 and W % 2 == 0
    out = np.empty((F, H // 2, W // 2, 2, 2, C), dtype=latent.dtype)
    for dy in range(2):
        for dx in range(2):
            out[:, :, :, dy, dx, :] = latent[:, dy::2, dx::2, :]
    return out.reshape(F * (H // 2) * (W // 2), 4 * C)


def unpatchify(tokens, F, H, W, C):
    """Inverse of patchify: [F * H/2 * W/2, 4C] -> [F, H, W, C]."""
    t = tokens.reshape(F, H // 2, W // 2, 2, 2, C)
    out = np.empty((F, H, W, C), dtype=tokens.dtype)
    for dy in range(2):
        for dx in range(2):
            out[:, dy::2, dx::2, :] = t[:, :, :, dy, dx, :]
    return out


class OracleEnds:
    """cfg: dict with dim, tok_h, tok_w, channels, freq_dim, eps.  weights: dict with END_KEYS and the
    timestep MLP (wt1, bt1, wt2, bt2)."""

    def __init__(self, cfg, weights, real="f64"):
        self.cfg = dict(cfg)
        self.ops = Ops(real)
        self.w = {k: self.ops.arr(v) for k, v in weights.items()}

    def embed(self, latent):
        """[F, 2*tok_h, 2*tok_w, C] latent -> [F * tok_h * tok_w, dim] tokens."""
        o = self.ops
        return o.linear(o.arr(patchify(np.asarray(latent))), self.w["w_pe"], self.w["b_pe"])

    def time_embedding(self, t):
        o, w = self.ops, self.w
        tau = o.sinusoid(t, self.cfg["freq_dim"])[None, :]
        return o.linear(o.silu(o.linear(tau, w["wt1"], w["bt1"])), w["wt2"], w["bt2"])[0]

    def head(self, x, t, n_frames):
        """[S, dim] tokens -> velocity in latent shape [F, 2*tok_h, 2*tok_w, C]."""
        o, c = self.ops, self.cfg
        e = self.time_embedding(t)
        shift, scale = self.w["m_head"][0] + e, self.w["m_head"][1] + e
        y = o.layernorm(o.arr(x), c["eps"], mul=1.0 + scale, add=shift)
        out = o.linear(y, self.w["w_head"], self.w["b_head"])
        return unpatchify(np.asarray(out), n_frames, 2 * c["tok_h"], 2 * c["tok_w"], c["channels"])


def euler_step(x, v, sigma, sigma_next):
    """x_{next} = x + (sigma_next - sigma) * v."""
    return np.asarray(x, dtype=np.float64) + (float(sigma_next) - float(sigma)) * np.asarray(v, dtype=np.float64)
