"""Pins of the oracle's primitives against things other than themselves: library routines used
as special-case checks, brute force in pure Python, closed forms and invariants."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle.ops import Ops


@pytest.fixture(scope="module")
def ops(oracle_built):
    return Ops("f64")


def rnd(*shape, seed=0):
    return np.random.default_rng(seed).standard_normal(shape)


def test_linear_matches_matmul_and_triple_loop(ops):
    x, W, b = rnd(5, 7), rnd(7, 3, seed=1), rnd(3, seed=2)
    y = ops.linear(x, W, b)
    np.testing.assert_allclose(y, x @ W + b, rtol=0, atol=1e-13)
    brute = [[sum(x[s, k] * W[k, n] for k in range(7)) + b[n] for n in range(3)] for s in range(5)]
    np.testing.assert_allclose(y, np.array(brute), rtol=0, atol=1e-13)
    # a transposed weight must not pass
    Wsq = rnd(7, 7, seed=3)
    assert np.abs(ops.linear(x, Wsq) - x @ Wsq.T).max() > 1e-3


def test_layernorm_matches_library(ops):
    x, mul, add = rnd(6, 32) * 3 + 1, rnd(32, seed=1), rnd(32, seed=2)
    ref = F.layer_norm(torch.from_numpy(x), (32,), torch.from_numpy(mul), torch.from_numpy(add), 1e-6).numpy()
    np.testing.assert_allclose(ops.layernorm(x, 1e-6, mul, add), ref, rtol=0, atol=1e-12)
    plain = ops.layernorm(x, 1e-6)
    np.testing.assert_allclose(plain.mean(1), 0, atol=1e-12)
    np.testing.assert_allclose(plain.var(1), 1, atol=1e-5)          # biased variance, eps-limited


def test_rmsnorm_closed_form(ops):
    x, g = rnd(4, 16), rnd(16, seed=1)
    y = ops.rmsnorm(x, g, 1e-6)
    ref = x / np.sqrt((x * x).mean(1, keepdims=True) + 1e-6) * g
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-13)
    # unit gain, zero eps: output has unit RMS over the full channel vector
    np.testing.assert_allclose(np.sqrt((ops.rmsnorm(x, np.ones(16), 0.0) ** 2).mean(1)), 1, atol=1e-13)


def test_gelu_silu(ops):
    x = np.linspace(-6, 6, 241)
    ref = F.gelu(torch.from_numpy(x), approximate="tanh").numpy()
    np.testing.assert_allclose(ops.gelu_tanh(x), ref, rtol=0, atol=1e-14)
    np.testing.assert_allclose(ops.gelu_tanh(x) - ops.gelu_tanh(-x), x, atol=1e-13)   # odd-part identity
    assert abs(ops.gelu_tanh(np.array([1.0]))[0] - 0.8411919906082768) < 1e-12
    # tanh form differs visibly from the erf form: the choice matters at fp32 tolerance
    assert np.abs(ref - F.gelu(torch.from_numpy(x)).numpy()).max() > 1e-4
    np.testing.assert_allclose(ops.silu(x), F.silu(torch.from_numpy(x)).numpy(), atol=1e-14)


def test_sinusoid(ops):
    t = 437.5
    s = ops.sinusoid(t, 256)
    np.testing.assert_allclose(s[:128] ** 2 + s[128:] ** 2, 1, atol=1e-13)
    assert abs(s[0] - math.cos(t)) < 1e-13 and abs(s[128] - math.sin(t)) < 1e-13      # w_0 = 1
    assert abs(s[64] - math.cos(t * 10000 ** -0.5)) < 1e-13                           # w_64 = 1e-2
    z = ops.sinusoid(0.0, 256)
    np.testing.assert_array_equal(z[:128], 1)
    np.testing.assert_array_equal(z[128:], 0)


def test_attention_rows_sum_to_one_and_brute_force(ops):
    S, L, h, d = 5, 9, 2, 4
    q, k, v = rnd(S, h * d), rnd(L, h * d, seed=1), rnd(L, h * d, seed=2)
    out, p = ops.attention(q, k, v, h, return_probs=True)
    np.testing.assert_allclose(p.sum(-1), 1, atol=1e-14)
    assert (p > 0).all()
    brute = np.zeros((S, h * d))
    for hd in range(h):
        for s in range(S):
            logits = [sum(q[s, hd * d + c] * k[j, hd * d + c] for c in range(d)) / math.sqrt(d) for j in range(L)]
            m = max(logits)
            e = [math.exp(z - m) for z in logits]
            for c in range(d):
                brute[s, hd * d + c] = sum(e[j] * v[j, hd * d + c] for j in range(L)) / sum(e)
    np.testing.assert_allclose(out, brute, atol=1e-13)
    # V := 1  =>  O = 1 ; key order is irrelevant
    np.testing.assert_allclose(ops.attention(q, k, np.ones_like(v), h), 1, atol=1e-14)
    perm = np.random.default_rng(5).permutation(L)
    np.testing.assert_allclose(ops.attention(q, k[perm], v[perm], h), out, atol=1e-13)


def test_attention_matches_library(ops):
    S, L, h, d = 17, 40, 3, 8
    q, k, v = rnd(S, h * d), rnd(L, h * d, seed=1), rnd(L, h * d, seed=2)
    tq, tk, tv = (torch.from_numpy(a).reshape(a.shape[0], h, d).transpose(0, 1) for a in (q, k, v))
    ref = F.scaled_dot_product_attention(tq, tk, tv).transpose(0, 1).reshape(S, h * d).numpy()
    np.testing.assert_allclose(ops.attention(q, k, v, h), ref, atol=1e-13)


def rope_args(n, seed=0, fmax=50, ymax=30, xmax=52):
    r = np.random.default_rng(seed)
    return r.integers(0, fmax, n), r.integers(0, ymax, n), r.integers(0, xmax, n)


@pytest.mark.parametrize("d", [64, 128])
def test_rope_invariants(ops, d):
    h, S = 2, 12
    x = rnd(S, h * d)
    zero = np.zeros(S, np.int32)
    np.testing.assert_array_equal(ops.rope3d(x, h, d, zero, zero, zero, 1e4), x)       # position 0 = identity
    pf, py, px = rope_args(S)
    y = ops.rope3d(x, h, d, pf, py, px, 1e4)
    pair = lambda a: (a.reshape(S, h, d // 2, 2) ** 2).sum(-1)
    np.testing.assert_allclose(pair(y), pair(x), atol=1e-12)                            # rotation keeps pair norms
    # channel split: frame axis owns the first c_f pairs of every head, rows the next c_h, columns the rest
    c_sp = d // 6
    c_f = d // 2 - 2 * c_sp
    assert (c_f, c_sp) == ((22, 21) if d == 128 else (12, 10))
    only_f = ops.rope3d(x, h, d, pf, zero, zero, 1e4).reshape(S, h, d // 2, 2)
    np.testing.assert_array_equal(only_f[:, :, c_f:], x.reshape(S, h, d // 2, 2)[:, :, c_f:])
    only_x = ops.rope3d(x, h, d, zero, zero, px, 1e4).reshape(S, h, d // 2, 2)
    np.testing.assert_array_equal(only_x[:, :, :c_f + c_sp], x.reshape(S, h, d // 2, 2)[:, :, :c_f + c_sp])
    # first pair of the frame group turns by exactly pf radians (theta^0 = 1)
    x0, x1 = x[:, 0], x[:, 1]
    np.testing.assert_allclose(y[:, 0], x0 * np.cos(pf) - x1 * np.sin(pf), atol=1e-12)
    np.testing.assert_allclose(y[:, 1], x0 * np.sin(pf) + x1 * np.cos(pf), atol=1e-12)
    # last pair of the frame group turns by pf * theta^(-(c_f-1)/c_f)
    a = pf * 1e4 ** (-(c_f - 1) / c_f)
    i = 2 * (c_f - 1)
    np.testing.assert_allclose(y[:, i], x[:, i] * np.cos(a) - x[:, i + 1] * np.sin(a), atol=1e-12)


def test_rope_relative_position(ops):
    """q.k after rotation depends only on position differences."""
    h, d = 1, 128
    q, k = rnd(1, d), rnd(1, d, seed=1)
    def dot(pq, pk):
        rq = ops.rope3d(q, h, d, [pq[0]], [pq[1]], [pq[2]], 1e4)
        rk = ops.rope3d(k, h, d, [pk[0]], [pk[1]], [pk[2]], 1e4)
        return float((rq * rk).sum())
    base = dot((3, 5, 7), (1, 2, 20))
    assert abs(dot((13, 9, 8), (11, 6, 21)) - base) < 1e-10
    assert abs(dot((3, 5, 7), (2, 2, 20)) - base) > 1e-3


def test_rope_matches_complex_form(ops):
    from ref_dit import rope_complex
    h, d, nf, f0, th, tw = 2, 64, 3, 5, 4, 6
    x = rnd(nf * th * tw, h * d)
    from oracle.stage import token_positions
    pf, py, px = token_positions(nf, f0, th, tw)
    ref = rope_complex(torch.from_numpy(x), h, d, nf, f0, th, tw, 1e4).numpy()
    np.testing.assert_allclose(ops.rope3d(x, h, d, pf, py, px, 1e4), ref, atol=1e-12)


def test_f32_build_tracks_f64(oracle_built):
    o32, o64 = Ops("f32"), Ops("f64")
    x, W = rnd(8, 64), rnd(64, 16, seed=1) * 0.1
    np.testing.assert_allclose(o32.linear(x, W), o64.linear(x, W), atol=1e-5)
    q, k, v = rnd(4, 32), rnd(10, 32, seed=1), rnd(10, 32, seed=2)
    np.testing.assert_allclose(o32.attention(q, k, v, 2), o64.attention(q, k, v, 2), atol=1e-5)
