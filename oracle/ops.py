"""ctypes bindings of the oracle's C++ primitives as numpy functions (TEST INFRASTRUCTURE).

Every function takes and returns C-contiguous numpy arrays of the oracle's
real type (float64 for `Ops("f64")`, float32 for `Ops("f32")`).
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_i64, _i32, _dbl = C.c_int64, C.c_int32, C.c_double


class Ops:
    def __init__(self, real: str = "f64"):
        assert real in ("f64", "f32")
        path = _build.lib_path(real)
        if not os.path.exists(path):
            _build.build()
        self.lib = C.CDLL(path)
        self.dtype = np.float64 if real == "f64" else np.float32
        self._creal = C.c_double if real == "f64" else C.c_float
        assert self.lib.orc_real_bytes() == np.dtype(self.dtype).itemsize
        P = C.c_void_p
        r = self._creal
        L = self.lib
        L.orc_linear.argtypes = [P, P, P, P, _i64, _i64, _i64]
        L.orc_layernorm.argtypes = [P, P, _i64, _i64, r, P, P]
        L.orc_rmsnorm.argtypes = [P, P, _i64, _i64, r, P]
        L.orc_rope3d.argtypes = [P, _i64, _i32, _i32, P, P, P, _dbl]
        L.orc_attention.argtypes = [P, P, P, P, _i64, _i64, _i32, _i32, P]
        L.orc_gelu_tanh.argtypes = [P, _i64]
        L.orc_silu.argtypes = [P, _i64]
        L.orc_sinusoid.argtypes = [_dbl, _i32, P]
        for f in (L.orc_linear, L.orc_layernorm, L.orc_rmsnorm, L.orc_rope3d, L.orc_attention,
                  L.orc_gelu_tanh, L.orc_silu, L.orc_sinusoid):
            f.restype = None

    # -- helpers ---------------------------------------------------------
    def arr(self, a):
        return np.ascontiguousarray(np.asarray(a), dtype=self.dtype)

    @staticmethod
    def _p(a):
        return None if a is None else a.ctypes.data_as(C.c_void_p)

    # -- primitives ------------------------------------------------------
    def linear(self, x, W, b=None):
        x, W = self.arr(x), self.arr(W)
        b = None if b is None else self.arr(b)
        S, K = x.shape
        K2, N = W.shape
        assert K == K2 and (b is None or b.shape == (N,))
        y = np.empty((S, N), self.dtype)
        self.lib.orc_linear(self._p(x), self._p(W), self._p(b), self._p(y), S, K, N)
        return y

    def layernorm(self, x, eps, mul=None, add=None):
        x = self.arr(x)
        S, D = x.shape
        mul = None if mul is None else self.arr(mul)
        add = None if add is None else self.arr(add)
        assert mul is None or mul.shape == (D,)
        assert add is None or add.shape == (D,)
        y = np.empty_like(x)
        self.lib.orc_layernorm(self._p(x), self._p(y), S, D, eps, self._p(mul), self._p(add))
        return y

    def rmsnorm(self, x, g, eps):
        x, g = self.arr(x), self.arr(g)
        S, D = x.shape
        assert g.shape == (D,)
        y = np.empty_like(x)
        self.lib.orc_rmsnorm(self._p(x), self._p(y), S, D, eps, self._p(g))
        return y

    def rope3d(self, x, n_heads, head_dim, pf, py, px, theta):
        """Returns the rotated copy of x[S, n_heads*head_dim]."""
        y = self.arr(x).copy()
        S, D = y.shape
        assert D == n_heads * head_dim and head_dim % 2 == 0
        pf, py, px = (np.ascontiguousarray(p, dtype=np.int32) for p in (pf, py, px))
        assert pf.shape == py.shape == px.shape == (S,)
        self.lib.orc_rope3d(self._p(y), S, n_heads, head_dim, self._p(pf), self._p(py), self._p(px), theta)
        return y

    def attention(self, q, k, v, n_heads, return_probs=False):
        q, k, v = self.arr(q), self.arr(k), self.arr(v)
        S, D = q.shape
        L = k.shape[0]
        assert k.shape == (L, D) and v.shape == (L, D) and D % n_heads == 0 and L > 0
        out = np.empty_like(q)
        probs = np.empty((n_heads, S, L), self.dtype) if return_probs else None
        self.lib.orc_attention(self._p(q), self._p(k), self._p(v), self._p(out), S, L, n_heads,
                               D // n_heads, self._p(probs))
        return (out, probs) if return_probs else out

    def gelu_tanh(self, x):
        y = self.arr(x).copy()
        self.lib.orc_gelu_tanh(self._p(y), y.size)
        return y

    def silu(self, x):
        y = self.arr(x).copy()
        self.lib.orc_silu(self._p(y), y.size)
        return y

    def sinusoid(self, t, freq_dim):
        out = np.empty((freq_dim,), self.dtype)
        self.lib.orc_sinusoid(float(t), freq_dim, self._p(out))
        return out
