// Bandwidth-bound kernels of the stage: type conversion, fused LayerNorm+modulate, q/k RMSNorm with
// 3D RoPE, V transposition, cache copies, the timestep-modulation vector and small utilities.
#include "kernels.h"

static inline int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// ---------------------------------------------------------------- conversions
// One thread per 8 elements (16 bytes of bf16, two 16-byte accesses of fp32) when pointers and length allow it.
template <typename T>
__global__ void k_to_f32(const T* __restrict__ in, float* __restrict__ out, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) out[i] = Elem<T>::ld(in + i);
}
template <typename T>
__global__ void k_from_f32(const float* __restrict__ in, T* __restrict__ out, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) Elem<T>::st(out + i, in[i]);
}
__global__ __launch_bounds__(256) void k_bf16_to_f32_x8(const uint4* __restrict__ in, float4* __restrict__ out, int64_t n8) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n8) return;
  const uint4 v = in[i];
  out[2 * i] = make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u),
                           __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xffff0000u));
  out[2 * i + 1] = make_float4(__uint_as_float(v.z << 16), __uint_as_float(v.z & 0xffff0000u),
                               __uint_as_float(v.w << 16), __uint_as_float(v.w & 0xffff0000u));
}
__global__ __launch_bounds__(256) void k_f32_to_bf16_x8(const float4* __restrict__ in, uint4* __restrict__ out, int64_t n8) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n8) return;
  const float4 a = in[2 * i], b = in[2 * i + 1];
  out[i] = make_uint4(pack_bf16x2(a.x, a.y), pack_bf16x2(a.z, a.w), pack_bf16x2(b.x, b.y), pack_bf16x2(b.z, b.w));
}
template <typename T> void launch_to_f32(const T* in, float* out, int64_t n, hipStream_t st) {
  if (n <= 0) return;
  if (sizeof(T) == 2 && n % 8 == 0 && (uintptr_t)in % 16 == 0 && (uintptr_t)out % 16 == 0) {
    k_bf16_to_f32_x8<<<cdiv(n / 8, 256), 256, 0, st>>>((const uint4*)in, (float4*)out, n / 8);
    return;
  }
  int grid = cdiv(n, 256); if (grid > 8192) grid = 8192;
  k_to_f32<T><<<grid, 256, 0, st>>>(in, out, n);
}
template <typename T> void launch_from_f32(const float* in, T* out, int64_t n, hipStream_t st) {
  if (n <= 0) return;
  if (sizeof(T) == 2 && n % 8 == 0 && (uintptr_t)in % 16 == 0 && (uintptr_t)out % 16 == 0) {
    k_f32_to_bf16_x8<<<cdiv(n / 8, 256), 256, 0, st>>>((const float4*)in, (uint4*)out, n / 8);
    return;
  }
  int grid = cdiv(n, 256); if (grid > 8192) grid = 8192;
  k_from_f32<T><<<grid, 256, 0, st>>>(in, out, n);
}
template void launch_to_f32<float>(const float*, float*, int64_t, hipStream_t);
template void launch_to_f32<bf16_t>(const bf16_t*, float*, int64_t, hipStream_t);
template void launch_from_f32<float>(const float*, float*, int64_t, hipStream_t);
template void launch_from_f32<bf16_t>(const float*, bf16_t*, int64_t, hipStream_t);

__global__ void k_mul_f32(const float* __restrict__ a, const float* __restrict__ b, float* __restrict__ out, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = a[i] * b[i];
}
void launch_mul_f32(const float* a, const float* b, float* out, int64_t n, hipStream_t st) {
  if (n > 0) k_mul_f32<<<cdiv(n, 256), 256, 0, st>>>(a, b, out, n);
}

__global__ void k_fill_zero(uint32_t* p, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = 0u;
}
void launch_fill_zero(void* p, size_t bytes, hipStream_t st) {   // bytes % 4 == 0
  int64_t n = (int64_t)(bytes / 4);
  if (n <= 0) return;
  int grid = cdiv(n, 256); if (grid > 16384) grid = 16384;
  k_fill_zero<<<grid, 256, 0, st>>>((uint32_t*)p, n);
}

// ---------------------------------------------------------------- LayerNorm + modulate
// NW wavefronts per row (1: a wavefront owns a row, 4 rows per block; 4: the block owns one row and the
// statistics meet in LDS); the row lives in registers (NCH float4 per lane), so x is read once.  Two-pass
// statistics (mean, then centred variance) in fp32, partial sums added in a fixed order.
// The row is read and the result written with non-temporal accesses: both are streamed once, and on this part
// a kernel that reads 4 and writes 2 bytes per element runs 1.4-1.7x faster that way (measured on flushed
// caches: 5120-wide rows 152 -> 89 us for 442 MB, 1536-wide rows 24 -> 15 us for 57 MB), faster than a plain
// conversion pass of the same bytes.  Wide rows gain another 25 % from four wavefronts per row (more rows in
// flight per compute unit, 5 instead of 20 outstanding loads per lane).
// xin != null: the row is read from xin (bf16) instead of x, and x receives its fp32 copy (the first
// LayerNorm of a stage, which thereby also fills the fp32 residual stream).
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
template <typename T, int NCH, int NW>
__global__ __launch_bounds__(256) void k_ln_modulate(float* __restrict__ x, const bf16_t* __restrict__ xin,
                                                     T* __restrict__ out, int64_t S, int D, float eps,
                                                     const float* __restrict__ mul,
                                                     const float* __restrict__ add, float plus) {
  static_assert(NW == 1 || NW == 2 || NW == 4, "wavefronts per row");
  constexpr int RPB = 4 / NW;                        // rows per block
  __shared__ float red[2][4];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int64_t row = (int64_t)blockIdx.x * RPB + w / NW;
  const int part = (w % NW) * 64 + lane;             // this lane's float4 slot inside a run of NW * 64 slots
  const bool live = row < S;                         // rows of a block end together only when NW > 1 shares them
  const int nvec = D >> 2;
  f32x4_t v[NCH];
  float sum = 0.f;
  if (live) {
    f32x4_t* xr = (f32x4_t*)(x + row * D);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int idx = i * (NW * 64) + part;
      if (idx < nvec) {
        if (xin) {
          const u32x2_t wv = __builtin_nontemporal_load((const u32x2_t*)(xin + row * D) + idx);
          v[i] = f32x4_t{bf16_to_f32((bf16_t)(wv.x & 0xffff)), bf16_to_f32((bf16_t)(wv.x >> 16)),
                         bf16_to_f32((bf16_t)(wv.y & 0xffff)), bf16_to_f32((bf16_t)(wv.y >> 16))};
          xr[idx] = v[i];
        } else {
          v[i] = __builtin_nontemporal_load(xr + idx);
        }
        sum += (v[i].x + v[i].y) + (v[i].z + v[i].w);
      }
      else v[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
  } else {
#pragma unroll
    for (int i = 0; i < NCH; ++i) v[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  }
  // sum over the row's NW wavefronts (consecutive wavefronts of the block), in wavefront order
  auto row_sum = [&](float part_sum, int slot) __attribute__((always_inline)) {
    float t = wave_sum(part_sum);
    if constexpr (NW > 1) {
      if (lane == 0) red[slot][w] = t;
      __syncthreads();
      t = 0.f;
#pragma unroll
      for (int i = 0; i < NW; ++i) t += red[slot][(w / NW) * NW + i];
    }
    return t;
  };
  const float mean = row_sum(sum, 0) / (float)D;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int idx = i * (NW * 64) + part;
    if (idx < nvec) {
      const float a = v[i].x - mean, b = v[i].y - mean, c = v[i].z - mean, d = v[i].w - mean;
      sq += (a * a + b * b) + (c * c + d * d);
    }
  }
  const float rstd = rsqrtf(row_sum(sq, 1) / (float)D + eps);
  if (!live) return;
  T* orow = out + row * D;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int idx = i * (NW * 64) + part;
    if (idx < nvec) {
      const float4 m = ((const float4*)mul)[idx];
      const float4 a = ((const float4*)add)[idx];
      const float r0 = (v[i].x - mean) * rstd * (m.x + plus) + a.x;
      const float r1 = (v[i].y - mean) * rstd * (m.y + plus) + a.y;
      const float r2 = (v[i].z - mean) * rstd * (m.z + plus) + a.z;
      const float r3 = (v[i].w - mean) * rstd * (m.w + plus) + a.w;
      if constexpr (sizeof(T) == 2) {
        u32x2_t pk; pk.x = pack_bf16x2(r0, r1); pk.y = pack_bf16x2(r2, r3);
        __builtin_nontemporal_store(pk, (u32x2_t*)orow + idx);
      } else {
        __builtin_nontemporal_store(f32x4_t{r0, r1, r2, r3}, (f32x4_t*)orow + idx);
      }
    }
  }
}
template <typename T>
void launch_ln_modulate(float* x, const bf16_t* xin, T* out, int64_t S, int D, float eps, const float* mul,
                        const float* add, int plus_one, hipStream_t st) {
  if (S <= 0) return;
  const float plus = plus_one ? 1.f : 0.f;
#define LN_CASE(NCH, NW) k_ln_modulate<T, NCH, NW><<<cdiv(S, 4 / NW), 256, 0, st>>>(x, xin, out, S, D, eps, mul, add, plus)
  if (D <= 256) LN_CASE(1, 1);
  else if (D <= 1536) LN_CASE(6, 1);
  else if (D <= 2048) LN_CASE(8, 1);
  else if (D <= 3072) LN_CASE(3, 4);
  else if (D <= 4096) LN_CASE(4, 4);
  else if (D <= 5120) LN_CASE(5, 4);
  else if (D <= 6144) LN_CASE(6, 4);
  else LN_CASE(8, 4);                                  // D <= 8192
#undef LN_CASE
}
template void launch_ln_modulate<float>(float*, const bf16_t*, float*, int64_t, int, float, const float*, const float*, int, hipStream_t);
template void launch_ln_modulate<bf16_t>(float*, const bf16_t*, bf16_t*, int64_t, int, float, const float*, const float*, int, hipStream_t);

// ---------------------------------------------------------------- RMSNorm over D + 3D RoPE, head-major output
// One wavefront per token and job (blockIdx.y: e.g. q and k of the same row), four tokens per block.  A lane
// owns VPL groups of 8 consecutive channels (one 16-byte access each for bf16), all loaded before the first
// use so that a wavefront keeps VPL KiB in flight, and kept in registers between the sum-of-squares pass and
// the normalise/rotate/store pass: the row is read once, and nothing but wavefront shuffles synchronises.
template <typename T> struct alignas(sizeof(T) * 8) Vec8 { T v[8]; };

template <typename T, int VPL>
__global__ __launch_bounds__(256) void k_norm_rope(const T* __restrict__ src, int64_t ld, int64_t S, int h, int d,
                                                   float eps, NormRopeJob<T> j0, NormRopeJob<T> j1,
                                                   RopeTables rt, int frame0, int tok_h, int tok_w) {
  const NormRopeJob<T> job = blockIdx.y == 0 ? j0 : j1;
  const int lane = threadIdx.x & 63;
  const int64_t s = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (s >= S) return;
  const int D = h * d, nvec = D >> 3;
  const Vec8<T>* row = (const Vec8<T>*)(src + s * ld + job.col);
  Vec8<T> raw[VPL];
#pragma unroll
  for (int i = 0; i < VPL; ++i) {
    const int vi = lane + i * 64;
    if (vi < nvec) raw[i] = row[vi];
  }
  float v[VPL][8];
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < VPL; ++i) {
    const int vi = lane + i * 64;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      v[i][e] = vi < nvec ? Elem<T>::ld(&raw[i].v[e]) : 0.f;
      sq += v[i][e] * v[i][e];
    }
  }
  const float r = rsqrtf(wave_sum(sq) / (float)D + eps) * job.out_scale;
  const int tok = tok_h * tok_w;
  const int f = frame0 + (int)(s / tok), rem = (int)(s % tok);
  const int y = rem / tok_w, x = rem % tok_w;
#pragma unroll
  for (int i = 0; i < VPL; ++i) {
    const int vi = lane + i * 64;
    if (vi < nvec) {
      const int c0 = vi * 8, head = c0 / d, p0 = (c0 % d) >> 1;        // first channel, its head, first pair in the head
      const float4 g0 = *(const float4*)(job.g + c0), g1 = *(const float4*)(job.g + c0 + 4);
      const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
      Vec8<T> o;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float a = v[i][2 * e] * r * gg[2 * e], b = v[i][2 * e + 1] * r * gg[2 * e + 1];
        if (job.rope) {
          const int pi = p0 + e;
          float2 cs;
          if (pi < rt.c_f) cs = rt.f[(int64_t)f * rt.c_f + pi];
          else if (pi < rt.c_f + rt.c_h) cs = rt.y[y * rt.c_h + (pi - rt.c_f)];
          else cs = rt.x[x * rt.c_w + (pi - rt.c_f - rt.c_h)];
          const float a2 = a * cs.x - b * cs.y, b2 = a * cs.y + b * cs.x;
          a = a2; b = b2;
        }
        Elem<T>::st(&o.v[2 * e], a);
        Elem<T>::st(&o.v[2 * e + 1], b);
      }
      *(Vec8<T>*)(job.dst + (int64_t)head * job.head_stride + (job.row0 + s) * d + (c0 % d)) = o;
    }
  }
}
template <typename T>
void launch_norm_rope(const T* src, int64_t ld, int64_t S, int h, int d, float eps, const NormRopeJob<T>* jobs,
                      int n_jobs, const RopeTables* rope, int frame0, int tok_h, int tok_w, hipStream_t st) {
  if (S <= 0 || n_jobs <= 0) return;
  RopeTables rt = rope ? *rope : RopeTables{nullptr, nullptr, nullptr, 0, 0, 0};
  NormRopeJob<T> j0 = jobs[0], j1 = jobs[n_jobs > 1 ? 1 : 0];
  if (!rope) { j0.rope = 0; j1.rope = 0; }
  const dim3 grid((unsigned)cdiv(S, 4), (unsigned)(n_jobs > 1 ? 2 : 1));
  const int th = tok_h > 0 ? tok_h : 1, tw = tok_w > 0 ? tok_w : 1;
  const int vpl = (h * d / 8 + 63) / 64;               // 16-byte groups per lane; dim <= 8192
#define NORM_ROPE_CASE(V) k_norm_rope<T, V><<<grid, 256, 0, st>>>(src, ld, S, h, d, eps, j0, j1, rt, frame0, th, tw)
  if (vpl <= 1) NORM_ROPE_CASE(1);
  else if (vpl <= 3) NORM_ROPE_CASE(3);
  else if (vpl <= 6) NORM_ROPE_CASE(6);
  else if (vpl <= 10) NORM_ROPE_CASE(10);
  else NORM_ROPE_CASE(16);
#undef NORM_ROPE_CASE
}
template void launch_norm_rope<float>(const float*, int64_t, int64_t, int, int, float, const NormRopeJob<float>*, int, const RopeTables*, int, int, int, hipStream_t);
template void launch_norm_rope<bf16_t>(const bf16_t*, int64_t, int64_t, int, int, float, const NormRopeJob<bf16_t>*, int, const RopeTables*, int, int, int, hipStream_t);

// ---------------------------------------------------------------- per-token rotation table of one block
// cs[s][i] = (cos, sin) of channel pair i at token s = (frame0 + s / (tok_h * tok_w), y, x), gathered from the
// three per-axis tables
__global__ void k_rope_tokens(RopeTables rt, int frame0, int tok_h, int tok_w, int64_t S, float2* __restrict__ cs) {
  const int half = rt.c_f + rt.c_h + rt.c_w;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= S * half) return;
  const int64_t s = i / half; const int pi = (int)(i % half);
  const int tok = tok_h * tok_w, rem = (int)(s % tok);
  const int f = frame0 + (int)(s / tok), y = rem / tok_w, x = rem % tok_w;
  float2 v;
  if (pi < rt.c_f) v = rt.f[(int64_t)f * rt.c_f + pi];
  else if (pi < rt.c_f + rt.c_h) v = rt.y[y * rt.c_h + (pi - rt.c_f)];
  else v = rt.x[x * rt.c_w + (pi - rt.c_f - rt.c_h)];
  cs[i] = v;
}
void launch_rope_tokens(const RopeTables& rt, int frame0, int tok_h, int tok_w, int64_t S, float2* cs, hipStream_t st) {
  if (S <= 0) return;
  k_rope_tokens<<<cdiv(S * (rt.c_f + rt.c_h + rt.c_w), 256), 256, 0, st>>>(rt, frame0, tok_h, tok_w, S, cs);
}

// ---------------------------------------------------------------- deferred RMSNorm of head-major bf16 rows
// k[head][row0 + s][:] *= rsqrt(sum_i ssq[i * stride + s] * inv_dim + eps) for every head: the row scale of an
// RMSNorm whose gains and rotation a GEMM epilogue has applied already.  One wavefront per token.
template <int VPL>
__global__ __launch_bounds__(256) void k_scale_rows(bf16_t* __restrict__ k, int64_t head_stride, int64_t row0, int64_t S,
                                                    int h, int d, const float* __restrict__ ssq, int np,
                                                    int64_t stride, float inv_dim, float eps) {
  const int lane = threadIdx.x & 63;
  const int64_t s = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (s >= S) return;
  const int nvec = (h * d) >> 3;
  uint4 raw[VPL];
#pragma unroll
  for (int i = 0; i < VPL; ++i) {
    const int c0 = (lane + i * 64) * 8;
    if (lane + i * 64 < nvec) raw[i] = *(const uint4*)(k + (int64_t)(c0 / d) * head_stride + (row0 + s) * d + c0 % d);
  }
  float sum = 0.f;
  for (int i = lane; i < np; i += 64) sum += ssq[i * stride + s];
  const float r = rsqrtf(wave_sum(sum) * inv_dim + eps);
#pragma unroll
  for (int i = 0; i < VPL; ++i) {
    const int c0 = (lane + i * 64) * 8;
    if (lane + i * 64 < nvec) {
      const uint32_t w[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
      uint32_t o[4];
#pragma unroll
      for (int e = 0; e < 4; ++e)
        o[e] = pack_bf16x2(bf16_to_f32((bf16_t)(w[e] & 0xffff)) * r, bf16_to_f32((bf16_t)(w[e] >> 16)) * r);
      *(uint4*)(k + (int64_t)(c0 / d) * head_stride + (row0 + s) * d + c0 % d) = make_uint4(o[0], o[1], o[2], o[3]);
    }
  }
}
void launch_scale_rows_bf16(bf16_t* k, int64_t head_stride, int64_t row0, int64_t S, int h, int d, const float* ssq,
                            int np, int64_t stride, float eps, hipStream_t st) {
  if (S <= 0) return;
  const int vpl = (h * d / 8 + 63) / 64;
  const float inv_dim = 1.f / (float)(h * d);
#define SCALE_ROWS_CASE(V) k_scale_rows<V><<<cdiv(S, 4), 256, 0, st>>>(k, head_stride, row0, S, h, d, ssq, np, stride, inv_dim, eps)
  if (vpl <= 1) SCALE_ROWS_CASE(1);
  else if (vpl <= 3) SCALE_ROWS_CASE(3);
  else if (vpl <= 6) SCALE_ROWS_CASE(6);
  else if (vpl <= 10) SCALE_ROWS_CASE(10);
  else SCALE_ROWS_CASE(16);
#undef SCALE_ROWS_CASE
}

// ---------------------------------------------------------------- V -> V^T (per head [d][L])
// 64 tokens x 64 channels through LDS: 16-byte reads along channels, 16-byte writes along tokens.
template <typename T>
__global__ __launch_bounds__(256) void k_v_transpose(const T* __restrict__ src, int64_t ld, int col, int64_t S,
                                                     int D, int d, T* __restrict__ vt, int64_t row_stride,
                                                     int64_t col0, int vec_ok) {
  __shared__ __align__(32) T tile[64][72];       // [channel][token], row padded, rows stay vector-aligned
  const int64_t s0 = (int64_t)blockIdx.x * 64;
  const int c0 = blockIdx.y * 64;
  const int t = threadIdx.x;
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int r = (t >> 3) + pass * 32, cc = (t & 7) * 8;
    const int64_t s = s0 + r;
    Vec8<T> x;
    if (s < S && c0 + cc < D) x = *(const Vec8<T>*)(src + s * ld + col + c0 + cc);
    else {
#pragma unroll
      for (int e = 0; e < 8; ++e) x.v[e] = (T)0;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) tile[cc + e][r] = x.v[e];
  }
  __syncthreads();
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int ch = (t >> 3) + pass * 32, tk = (t & 7) * 8;
    const int c = c0 + ch;
    const int64_t s = s0 + tk;
    if (c < D && s < S) {
      T* o = vt + (int64_t)c * row_stride + col0 + s;     // channel c = head*d + cc: row c of [h*d][row_stride]
      if (vec_ok && s + 8 <= S) *(Vec8<T>*)o = *(const Vec8<T>*)&tile[ch][tk];
      else for (int e = 0; e < 8 && s + e < S; ++e) o[e] = tile[ch][tk + e];
    }
  }
}
template <typename T>
void launch_v_transpose(const T* src, int64_t ld, int col, int64_t S, int h, int d, T* vt,
                        int64_t row_stride, int64_t col0, hipStream_t st) {
  if (S <= 0) return;
  dim3 grid(cdiv(S, 64), cdiv(h * d, 64));
  const int vec_ok = (col0 % 8 == 0) && (row_stride % 8 == 0) && ((uintptr_t)vt % (8 * sizeof(T)) == 0);
  k_v_transpose<T><<<grid, 256, 0, st>>>(src, ld, col, S, h * d, d, vt, row_stride, col0, vec_ok);
}
template void launch_v_transpose<float>(const float*, int64_t, int, int64_t, int, int, float*, int64_t, int64_t, hipStream_t);
template void launch_v_transpose<bf16_t>(const bf16_t*, int64_t, int, int64_t, int, int, bf16_t*, int64_t, int64_t, hipStream_t);

// ---------------------------------------------------------------- strided row copy (feature-cache hand-over)
// Rows are copied in 16-byte pieces when src, dst, strides and length allow it.
template <typename T, typename V>
__global__ void k_copy2d(const T* __restrict__ src, int64_t src_stride, T* __restrict__ dst,
                         int64_t dst_stride, int64_t len_v) {
  const V* s = (const V*)(src + (int64_t)blockIdx.y * src_stride);
  V* d = (V*)(dst + (int64_t)blockIdx.y * dst_stride);
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < len_v; i += stride) d[i] = s[i];
}
template <typename T>
void launch_copy2d(const T* src, int64_t src_stride, T* dst, int64_t dst_stride, int64_t rows,
                   int64_t len, hipStream_t st) {
  if (rows <= 0 || len <= 0) return;
  const int per = 16 / (int)sizeof(T);
  const bool vec = ((uintptr_t)src % 16 == 0) && ((uintptr_t)dst % 16 == 0) && (src_stride % per == 0) &&
                   (dst_stride % per == 0) && (len % per == 0);
  // rows can exceed the grid.y limit only for absurd shapes; split defensively
  for (int64_t r0 = 0; r0 < rows; r0 += 32768) {
    const int64_t nr = rows - r0 < 32768 ? rows - r0 : 32768;
    if (vec) {
      const int64_t lv = len / per;
      int gx = cdiv(lv, 256); if (gx > 64) gx = 64;
      k_copy2d<T, uint4><<<dim3(gx, (unsigned)nr), 256, 0, st>>>(src + r0 * src_stride, src_stride,
                                                                 dst + r0 * dst_stride, dst_stride, lv);
    } else {
      int gx = cdiv(len, 256); if (gx > 64) gx = 64;
      k_copy2d<T, T><<<dim3(gx, (unsigned)nr), 256, 0, st>>>(src + r0 * src_stride, src_stride,
                                                             dst + r0 * dst_stride, dst_stride, len);
    }
  }
}
template void launch_copy2d<float>(const float*, int64_t, float*, int64_t, int64_t, int64_t, hipStream_t);
template void launch_copy2d<bf16_t>(const bf16_t*, int64_t, bf16_t*, int64_t, int64_t, int64_t, hipStream_t);

// ---------------------------------------------------------------- weight repack: [K,N] -> [Npad,K]
template <typename T>
__global__ __launch_bounds__(256) void k_transpose_pad(const T* __restrict__ in, int64_t K, int64_t N,
                                                       T* __restrict__ out, int64_t Npad) {
  __shared__ T tile[64][65];
  const int64_t k0 = (int64_t)blockIdx.x * 64, n0 = (int64_t)blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int r = ty; r < 64; r += 4) {
    const int64_t k = k0 + r, n = n0 + tx;
    tile[r][tx] = (k < K && n < N) ? in[k * N + n] : (T)0;
  }
  __syncthreads();
  for (int r = ty; r < 64; r += 4) {
    const int64_t n = n0 + r, k = k0 + tx;
    if (n < Npad && k < K) out[n * K + k] = tile[tx][r];
  }
}
template <typename T>
void launch_transpose_pad(const T* in, int64_t K, int64_t N, T* out, int64_t Npad, hipStream_t st) {
  dim3 grid(cdiv(K, 64), cdiv(Npad, 64));
  k_transpose_pad<T><<<grid, 256, 0, st>>>(in, K, N, out, Npad);
}
template void launch_transpose_pad<float>(const float*, int64_t, int64_t, float*, int64_t, hipStream_t);
template void launch_transpose_pad<bf16_t>(const bf16_t*, int64_t, int64_t, bf16_t*, int64_t, hipStream_t);

// ---------------------------------------------------------------- timestep modulation vector
__global__ void k_sinusoid(float t, int freq_dim, float* out) {
  const int half = freq_dim >> 1;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= half) return;
  const double w = pow(10000.0, -(double)i / (double)half);
  const double a = (double)t * w;
  out[i] = (float)cos(a);
  out[half + i] = (float)sin(a);
}
void launch_sinusoid(float t, int freq_dim, float* out, hipStream_t st) {
  k_sinusoid<<<cdiv(freq_dim / 2, 64), 64, 0, st>>>(t, freq_dim, out);
}

// Matrix-vector products of the timestep MLP.  A block owns 64 output columns and one of gridDim.y slices of the
// K rows; its 16 wavefronts each take every 16th row of the slice (coalesced 64-column reads) and the partial
// sums meet in LDS.  The block writes its slice's partial result y[slice][n] without bias: whoever consumes the
// vector adds the slices up in index order (so the result does not depend on timing) together with the bias.
// The input is such a sliced vector itself: x[k] = act(sum_p x[p][k] + xbias[k]).
template <typename T>
__global__ __launch_bounds__(1024) void k_gemv(const float* __restrict__ x, int x_parts, int x_stride,
                                               const T* __restrict__ xbias, int K, const T* __restrict__ W, int N,
                                               int silu_in, float* __restrict__ y) {
  extern __shared__ float xs[];            // this slice's activations, then 16 x 64 partial sums
  const int KS = gridDim.y, ks = blockIdx.y;
  const int k0 = (int)((int64_t)K * ks / KS), Kb = (int)((int64_t)K * (ks + 1) / KS) - k0;
  float* red = xs + Kb;
  for (int k = threadIdx.x; k < Kb; k += 1024) {
    float v = xbias ? Elem<T>::ld(xbias + k0 + k) : 0.f;
    for (int p = 0; p < x_parts; ++p) v += x[(int64_t)p * x_stride + k0 + k];
    xs[k] = silu_in ? v / (1.0f + expf(-v)) : v;
  }
  __syncthreads();
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int n = blockIdx.x * 64 + tx;
  const T* Wb = W + (int64_t)k0 * N;
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  if (n < N) {
    int k = ty;
    for (; k + 48 < Kb; k += 64) {
      a0 += xs[k] * Elem<T>::ld(Wb + (int64_t)k * N + n);
      a1 += xs[k + 16] * Elem<T>::ld(Wb + (int64_t)(k + 16) * N + n);
      a2 += xs[k + 32] * Elem<T>::ld(Wb + (int64_t)(k + 32) * N + n);
      a3 += xs[k + 48] * Elem<T>::ld(Wb + (int64_t)(k + 48) * N + n);
    }
    for (; k < Kb; k += 16) a0 += xs[k] * Elem<T>::ld(Wb + (int64_t)k * N + n);
  }
  red[ty * 64 + tx] = (a0 + a1) + (a2 + a3);
  __syncthreads();
  if (ty == 0 && n < N) {
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) sum += red[i * 64 + tx];
    y[(int64_t)ks * N + n] = sum;
  }
}
int gemv_slices(int K, int N) {
  int ks = (256 + cdiv(N, 64) - 1) / cdiv(N, 64);     // enough blocks for the 256 CUs
  if (ks > GEMV_MAX_SLICES) ks = GEMV_MAX_SLICES;
  while (ks > 1 && K / ks < 64) --ks;
  return ks < 1 ? 1 : ks;
}
template <typename T>
void launch_gemv(const float* x, int x_parts, int x_stride, const T* xbias, int K, const T* W, int N, int silu_in,
                 float* y, hipStream_t st) {
  const int ks = gemv_slices(K, N);
  k_gemv<T><<<dim3(cdiv(N, 64), ks), 1024, (size_t)(cdiv(K, ks) + 1 + 1024) * sizeof(float), st>>>(
      x, x_parts, x_stride, xbias, K, W, N, silu_in, y);
}
template void launch_gemv<float>(const float*, int, int, const float*, int, const float*, int, int, float*, hipStream_t);
template void launch_gemv<bf16_t>(const float*, int, int, const bf16_t*, int, const bf16_t*, int, int, float*, hipStream_t);

// mod[l, i] = mtab[l, i] + sum_p e[p][i] + bias[i]: a sliced vector (see k_gemv) added to every row of a table
template <typename T>
__global__ void k_mod_add(const float* __restrict__ mtab, const float* __restrict__ e, int parts,
                          const T* __restrict__ bias, float* __restrict__ mod, int L, int n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)L * n) return;
  const int c = (int)(i % n);
  float v = bias ? Elem<T>::ld(bias + c) : 0.f;
  for (int p = 0; p < parts; ++p) v += e[(int64_t)p * n + c];
  mod[i] = mtab[i] + v;
}
template <typename T>
void launch_mod_add(const float* mtab, const float* e, int parts, const T* bias, float* mod, int L, int n, hipStream_t st) {
  k_mod_add<T><<<cdiv((int64_t)L * n, 256), 256, 0, st>>>(mtab, e, parts, bias, mod, L, n);
}
template void launch_mod_add<float>(const float*, const float*, int, const float*, float*, int, int, hipStream_t);
template void launch_mod_add<bf16_t>(const float*, const float*, int, const bf16_t*, float*, int, int, hipStream_t);

// cos/sin of pos * theta^(-i/pairs), angles in double
__global__ void k_rope_table(float2* tab, int n_pos, int pairs, float theta) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_pos * pairs) return;
  const int pos = i / pairs, j = i % pairs;
  const double ang = (double)pos * pow((double)theta, -(double)j / (double)pairs);
  tab[i] = make_float2((float)cos(ang), (float)sin(ang));
}
void launch_rope_table(float2* tab, int n_pos, int pairs, float theta, hipStream_t st) {
  if (n_pos * pairs <= 0) return;
  k_rope_table<<<cdiv((int64_t)n_pos * pairs, 256), 256, 0, st>>>(tab, n_pos, pairs, theta);
}

// ---------------------------------------------------------------- test-hook gathers (head-major -> token-major fp32)
template <typename T>
__global__ void k_gather_heads(const T* __restrict__ src, int64_t head_stride, int64_t row0, int64_t S,
                               int h, int d, float* __restrict__ dst) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int D = h * d;
  if (i >= S * D) return;
  const int64_t s = i / D; const int c = (int)(i % D);
  dst[i] = Elem<T>::ld(src + (int64_t)(c / d) * head_stride + (row0 + s) * d + (c % d));
}
template <typename T>
void launch_gather_heads(const T* src, int64_t head_stride, int64_t row0, int64_t S, int h, int d,
                         float* dst, hipStream_t st) {
  if (S <= 0) return;
  k_gather_heads<T><<<cdiv(S * h * d, 256), 256, 0, st>>>(src, head_stride, row0, S, h, d, dst);
}
// the queries as the bf16 attention kernel uses them when their RMSNorm is deferred: same sums, same rounding
__global__ void k_gather_heads_qnorm(const bf16_t* __restrict__ src, int64_t head_stride, int64_t S, int h, int d,
                                     AttnQNorm qn, float* __restrict__ dst) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int D = h * d;
  if (i >= S * D) return;
  const int64_t s = i / D; const int c = (int)(i % D);
  float even = 0.f, odd = 0.f;
  for (int j = 0; j < qn.np; j += 2) even += qn.ssq[j * qn.stride + s];
  for (int j = 1; j < qn.np; j += 2) odd += qn.ssq[j * qn.stride + s];
  const float r = rsqrtf((even + odd) * qn.inv_dim + qn.eps) * qn.scale;
  dst[i] = bf16_to_f32(f32_to_bf16(bf16_to_f32(src[(int64_t)(c / d) * head_stride + s * d + (c % d)]) * r));
}
void launch_gather_heads_qnorm(const bf16_t* src, int64_t head_stride, int64_t S, int h, int d, const AttnQNorm& qn,
                               float* dst, hipStream_t st) {
  if (S <= 0) return;
  k_gather_heads_qnorm<<<cdiv(S * h * d, 256), 256, 0, st>>>(src, head_stride, S, h, d, qn, dst);
}
template void launch_gather_heads<float>(const float*, int64_t, int64_t, int64_t, int, int, float*, hipStream_t);
template void launch_gather_heads<bf16_t>(const bf16_t*, int64_t, int64_t, int64_t, int, int, float*, hipStream_t);

template <typename T>
__global__ void k_gather_vt(const T* __restrict__ vt, int64_t row_stride, int64_t col0, int64_t S, int h,
                            int d, float* __restrict__ dst) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int D = h * d;
  if (i >= S * D) return;
  const int64_t s = i / D; const int c = (int)(i % D);
  dst[i] = Elem<T>::ld(vt + (int64_t)c * row_stride + col0 + s);
}
template <typename T>
void launch_gather_vt(const T* vt, int64_t row_stride, int64_t col0, int64_t S, int h, int d, float* dst,
                      hipStream_t st) {
  if (S <= 0) return;
  k_gather_vt<T><<<cdiv(S * h * d, 256), 256, 0, st>>>(vt, row_stride, col0, S, h, d, dst);
}
template void launch_gather_vt<float>(const float*, int64_t, int64_t, int64_t, int, int, float*, hipStream_t);
template void launch_gather_vt<bf16_t>(const bf16_t*, int64_t, int64_t, int64_t, int, int, float*, hipStream_t);

// ---------------------------------------------------------------- coordinated noise initialisation: frame gather
// out[f, :] = pool[index[f], :] in 16-byte vectors; a frame whose index is out of range is written as zeros
__global__ __launch_bounds__(256) void k_gather_frames(const uint4* __restrict__ pool, int pool_frames,
                                                       int64_t frame_vecs, const int32_t* __restrict__ index,
                                                       uint4* __restrict__ out) {
  const int f = blockIdx.y;
  const int src = index[f];
  const bool ok = src >= 0 && src < pool_frames;
  const uint4* s = pool + (int64_t)(ok ? src : 0) * frame_vecs;
  uint4* d = out + (int64_t)f * frame_vecs;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < frame_vecs; i += (int64_t)gridDim.x * 256)
    d[i] = ok ? s[i] : make_uint4(0, 0, 0, 0);
}
void launch_gather_frames(const void* pool, int pool_frames, int64_t frame_bytes, const int32_t* index,
                          int n_frames, void* out, hipStream_t st) {
  if (n_frames <= 0 || frame_bytes <= 0) return;
  const int64_t vecs = frame_bytes / 16;
  int64_t bx = cdiv(vecs, 256 * 4);                 // 4 vectors per thread
  if (bx < 1) bx = 1;
  if (bx > 4096) bx = 4096;
  k_gather_frames<<<dim3((unsigned)bx, (unsigned)n_frames), 256, 0, st>>>((const uint4*)pool, pool_frames, vecs, index, (uint4*)out);
}
