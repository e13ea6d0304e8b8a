// fp32 softmax attention for the DP_F32 path.  One wavefront per (head, query); keys are taken 64 at
// a time (one per lane) with an online softmax.  Each lane keeps a private partial output over its
// own keys; the partials are summed across the wavefront once at the end.
#include "kernels.h"

template <int HD>
__global__ __launch_bounds__(256) void k_attn_f32(const float* __restrict__ q, int64_t q_head_stride,
                                                  const float* __restrict__ k, int64_t k_head_stride,
                                                  int64_t k_row0, const float* __restrict__ vt,
                                                  int64_t vt_row_stride, int64_t S, int64_t L,
                                                  float* __restrict__ out, int64_t ldo, float scale) {
  __shared__ float qs[4][HD];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t s = (int64_t)blockIdx.x * 4 + w;
  const int head = blockIdx.y;
  if (s >= S) return;                       // whole wavefront leaves together; no block barrier below
  const float* qrow = q + (int64_t)head * q_head_stride + s * HD;
  for (int c = lane; c < HD; c += 64) qs[w][c] = qrow[c] * scale;
  __builtin_amdgcn_wave_barrier();
  const float* kh = k + (int64_t)head * k_head_stride + k_row0 * HD;
  const float* vh = vt + (int64_t)head * HD * vt_row_stride + k_row0;
  float acc[HD];
#pragma unroll
  for (int c = 0; c < HD; ++c) acc[c] = 0.f;
  float m = -INFINITY, l = 0.f;             // running max (wave-uniform) and this lane's partial sum
  for (int64_t j0 = 0; j0 < L; j0 += 64) {
    const int64_t j = j0 + lane;
    float sc = -INFINITY;
    if (j < L) {
      const float4* kr = (const float4*)(kh + j * HD);
      float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;
#pragma unroll
      for (int c = 0; c < HD / 4; ++c) {
        const float4 kv = kr[c];
        d0 = fmaf(qs[w][4 * c], kv.x, d0); d1 = fmaf(qs[w][4 * c + 1], kv.y, d1);
        d2 = fmaf(qs[w][4 * c + 2], kv.z, d2); d3 = fmaf(qs[w][4 * c + 3], kv.w, d3);
      }
      sc = (d0 + d1) + (d2 + d3);
    }
    const float mnew = fmaxf(m, wave_max(sc));
    const float alpha = expf(m - mnew);     // 0 on the first chunk (m = -inf)
    const float p = (j < L) ? expf(sc - mnew) : 0.f;
    l = l * alpha + p;
    if (j < L) {
#pragma unroll
      for (int c = 0; c < HD; ++c) acc[c] = fmaf(p, vh[(int64_t)c * vt_row_stride + j], acc[c] * alpha);
    } else {
#pragma unroll
      for (int c = 0; c < HD; ++c) acc[c] *= alpha;
    }
    m = mnew;
  }
  const float inv = 1.f / wave_sum(l);
  float* o = out + s * ldo + head * HD;
#pragma unroll
  for (int c = 0; c < HD; ++c) {
    const float t = wave_sum(acc[c]);
    if (lane == (c & 63)) o[c] = t * inv;
  }
}

void launch_attn_f32(const float* q, int64_t q_head_stride, const float* k, int64_t k_head_stride,
                     int64_t k_row0, const float* vt, int64_t vt_row_stride, int64_t S, int64_t L,
                     int h, int d, float* out, int64_t ldo, hipStream_t st) {
  if (S <= 0 || L <= 0) return;
  dim3 grid((unsigned)((S + 3) / 4), (unsigned)h);
  const float scale = 1.0f / sqrtf((float)d);
  if (d == 64)
    k_attn_f32<64><<<grid, 256, 0, st>>>(q, q_head_stride, k, k_head_stride, k_row0, vt, vt_row_stride, S, L, out, ldo, scale);
  else
    k_attn_f32<128><<<grid, 256, 0, st>>>(q, q_head_stride, k, k_head_stride, k_row0, vt, vt_row_stride, S, L, out, ldo, scale);
}
