// CPU oracle primitives for the block-wise denoising stage (TEST INFRASTRUCTURE).
//
// Plain, slow, loop-level definitions of every operator a DiT stage applies to
// one frame block (paper Sec. 2 Eq. 1, Sec. 3.2): linear maps, LayerNorm,
// RMSNorm, 3D rotary embedding, softmax attention over an explicit key/value
// list, tanh-GELU, SiLU and the sinusoidal timestep features.  The paper
// treats the DiT layer as a black box; the operator definitions here are the
// build's stated readings of a Wan-shaped layer.
//
// No blocking, no fusion, no reordering beyond the textbook definition.
// OpenMP is used only across independent rows / heads.  The arithmetic type is
// `real` (double unless built with -DORC_REAL=float).  This file shares no
// code with the GPU library and must never be linked into it.
#include <cmath>
#include <cstdint>
#include <vector>

#ifndef ORC_REAL
#define ORC_REAL double
#endif
typedef ORC_REAL real;

extern "C" {

int orc_real_bytes(void) { return (int)sizeof(real); }

// y[s,n] = sum_k x[s,k] * W[k,n] + b[n]      (W row-major [K,N]; b may be null)
void orc_linear(const real* x, const real* W, const real* b, real* y,
                int64_t S, int64_t K, int64_t N) {
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < S; ++s) {
    real* yr = y + s * N;
    for (int64_t n = 0; n < N; ++n) yr[n] = b ? b[n] : (real)0;
    for (int64_t k = 0; k < K; ++k) {
      const real xv = x[s * K + k];
      const real* wr = W + k * N;
      for (int64_t n = 0; n < N; ++n) yr[n] += xv * wr[n];
    }
  }
}

// LayerNorm without learned affine, biased variance, followed by a per-channel
// multiply and add:  y = (x - mean) / sqrt(var + eps) * mul + add.
// mul / add may be null (treated as 1 / 0).
void orc_layernorm(const real* x, real* y, int64_t S, int64_t D, real eps,
                   const real* mul, const real* add) {
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < S; ++s) {
    const real* xr = x + s * D;
    real mean = 0;
    for (int64_t c = 0; c < D; ++c) mean += xr[c];
    mean /= (real)D;
    real var = 0;
    for (int64_t c = 0; c < D; ++c) var += (xr[c] - mean) * (xr[c] - mean);
    var /= (real)D;
    const real rstd = (real)1 / std::sqrt(var + eps);
    for (int64_t c = 0; c < D; ++c) {
      real v = (xr[c] - mean) * rstd;
      if (mul) v *= mul[c];
      if (add) v += add[c];
      y[s * D + c] = v;
    }
  }
}

// RMSNorm over the whole channel vector: y = x / sqrt(mean(x^2) + eps) * g
void orc_rmsnorm(const real* x, real* y, int64_t S, int64_t D, real eps, const real* g) {
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < S; ++s) {
    const real* xr = x + s * D;
    real ms = 0;
    for (int64_t c = 0; c < D; ++c) ms += xr[c] * xr[c];
    ms /= (real)D;
    const real r = (real)1 / std::sqrt(ms + eps);
    for (int64_t c = 0; c < D; ++c) y[s * D + c] = xr[c] * r * g[c];
  }
}

// 3D rotary embedding, in place on x[S, h*d].  Token s sits at integer
// position (pf[s], py[s], px[s]).  Inside each head the d/2 channel pairs
// (2i, 2i+1) are split into three consecutive groups [c_f | c_h | c_w] with
// c_h = c_w = floor(d/6), c_f = d/2 - 2*floor(d/6).  Pair i of a group with c
// pairs on axis position p is rotated by the angle p * theta^(-i/c):
//   (x0, x1) -> (x0 cos - x1 sin, x0 sin + x1 cos).
void orc_rope3d(real* x, int64_t S, int32_t h, int32_t d, const int32_t* pf,
                const int32_t* py, const int32_t* px, double theta) {
  const int32_t half = d / 2;
  const int32_t c_h = d / 6, c_w = d / 6, c_f = half - 2 * (d / 6);
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < S; ++s) {
    for (int32_t hd = 0; hd < h; ++hd) {
      real* v = x + s * (int64_t)h * d + (int64_t)hd * d;
      for (int32_t i = 0; i < half; ++i) {
        double pos; int32_t j, c;
        if (i < c_f) { pos = pf[s]; j = i; c = c_f; }
        else if (i < c_f + c_h) { pos = py[s]; j = i - c_f; c = c_h; }
        else { pos = px[s]; j = i - c_f - c_h; c = c_w; }
        const double ang = pos * std::pow(theta, -(double)j / (double)c);
        const real cs = (real)std::cos(ang), sn = (real)std::sin(ang);
        const real x0 = v[2 * i], x1 = v[2 * i + 1];
        v[2 * i] = x0 * cs - x1 * sn;
        v[2 * i + 1] = x0 * sn + x1 * cs;
      }
    }
  }
}

// Multi-head softmax attention, no mask.  q[S, h*d], k[L, h*d], v[L, h*d],
// out[S, h*d]; head hd owns channels [hd*d, (hd+1)*d).  For every head and
// query: p_j = softmax_j(q . k_j / sqrt(d)),  out = sum_j p_j v_j.
// probs (optional) receives p as [h, S, L].
void orc_attention(const real* q, const real* k, const real* v, real* out,
                   int64_t S, int64_t L, int32_t h, int32_t d, real* probs) {
  const int64_t D = (int64_t)h * d;
  const real scale = (real)1 / std::sqrt((real)d);
#pragma omp parallel for collapse(2) schedule(static)
  for (int32_t hd = 0; hd < h; ++hd) {
    for (int64_t s = 0; s < S; ++s) {
      std::vector<real> p((size_t)L);
      const real* qv = q + s * D + (int64_t)hd * d;
      real mx = -INFINITY;
      for (int64_t j = 0; j < L; ++j) {
        const real* kv = k + j * D + (int64_t)hd * d;
        real dot = 0;
        for (int32_t c = 0; c < d; ++c) dot += qv[c] * kv[c];
        p[j] = dot * scale;
        if (p[j] > mx) mx = p[j];
      }
      real sum = 0;
      for (int64_t j = 0; j < L; ++j) { p[j] = std::exp(p[j] - mx); sum += p[j]; }
      for (int64_t j = 0; j < L; ++j) p[j] /= sum;
      real* o = out + s * D + (int64_t)hd * d;
      for (int32_t c = 0; c < d; ++c) o[c] = 0;
      for (int64_t j = 0; j < L; ++j) {
        const real* vv = v + j * D + (int64_t)hd * d;
        for (int32_t c = 0; c < d; ++c) o[c] += p[j] * vv[c];
      }
      if (probs) {
        real* pr = probs + ((int64_t)hd * S + s) * L;
        for (int64_t j = 0; j < L; ++j) pr[j] = p[j];
      }
    }
  }
}

// tanh-approximate GELU: 0.5 x (1 + tanh( sqrt(2/pi) (x + 0.044715 x^3) )), in place.
void orc_gelu_tanh(real* x, int64_t n) {
  const real c = (real)0.79788456080286535587989211986876;  // sqrt(2/pi)
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    const real v = x[i];
    x[i] = (real)0.5 * v * ((real)1 + std::tanh(c * (v + (real)0.044715 * v * v * v)));
  }
}

// SiLU: x * sigmoid(x), in place.
void orc_silu(real* x, int64_t n) {
  for (int64_t i = 0; i < n; ++i) x[i] = x[i] / ((real)1 + std::exp(-x[i]));
}

// Sinusoidal timestep features, cosine half first:
//   out[i] = cos(t * w_i), out[half + i] = sin(t * w_i),  w_i = 10000^(-i/half), half = freq_dim/2.
void orc_sinusoid(double t, int32_t freq_dim, real* out) {
  const int32_t half = freq_dim / 2;
  for (int32_t i = 0; i < half; ++i) {
    const double w = std::pow(10000.0, -(double)i / (double)half);
    out[i] = (real)std::cos(t * w);
    out[half + i] = (real)std::sin(t * w);
  }
}

}  // extern "C"
