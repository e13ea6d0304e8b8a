// Shared device helpers of libdualparal (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

typedef uint16_t bf16_t;   // storage of a bfloat16: the upper half of an IEEE float

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float ld(const float* p) { return *p; }
  static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float ld(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void st(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// Barrier that publishes an LDS tile which the block's wavefronts loaded together with direct
// global -> LDS loads.  The compiler orders such a load only against the issuing wavefront's own later LDS
// reads, not against a barrier, so every wavefront first waits for its outstanding vector-memory loads
// itself (s_waitcnt vmcnt(0); the other counters are left alone) and then joins the barrier.
__device__ __forceinline__ void tile_barrier() {
  __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt = 0, expcnt = 7 and lgkmcnt = 15 (no wait)
  __syncthreads();
}


// ---- hand-scheduled loops: compile-time unrolling, LDS reads the compiler does not track, exact waits
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{}) in this order
template <int N, typename F> __device__ __forceinline__ void static_for(F&& f) {
  if constexpr (N > 0) { static_for<N - 1>(f); f(std::integral_constant<int, N - 1>{}); }
}
// wait until at most C of this wavefront's LDS operations are outstanding (the other counters are left alone);
// LDS operations complete in order, so everything but the C newest has then landed
template <int C> __device__ __forceinline__ void lds_wait() {
  if constexpr (C < 15) __builtin_amdgcn_s_waitcnt(0xC07F | (C << 8));
}
// 16 bytes at LDS byte address addr + OFF through inline assembly: the compiler neither moves it nor waits for
// it; the caller does (lds_wait) before the first use of the result
template <int OFF> __device__ __forceinline__ u32x4 lds_read16_raw(uint32_t addr) {
  u32x4 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(v) : "v"(addr), "n"(OFF));
  return v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

__device__ __forceinline__ float gelu_tanh_f(float v) {
  const float c = 0.7978845608028654f;
  return 0.5f * v * (1.0f + tanhf(c * (v + 0.044715f * v * v * v)));
}
__device__ __forceinline__ float silu_f(float v) { return v / (1.0f + __expf(-v)); }

// GEMM epilogue selector (shared by the fp32 and the bf16 GEMM kernels; EPI_HEADS is bf16 only)
enum { EPI_STORE = 0, EPI_GELU = 1, EPI_RESID = 2, EPI_HEADS = 3 };

struct RopeTables {            // cos/sin pairs: tab[pos][pair] = (cos, sin)
  const float2* f; const float2* y; const float2* x;
  int c_f, c_h, c_w;           // pairs per axis
};

// EPI_HEADS: the output columns are up to three sections of `dim` columns each (e.g. q | k | v of a fused
// projection); a section is written per attention head instead of row-major.
struct HeadSection {
  void* dst;               // plain: [dim / head_dim][..][head_dim], element (head, row0 + m, c);
                           // transposed: [dim][ld], element (channel, row0 + m)
  int64_t ld;              // plain: elements between heads; transposed: elements between channels
  int64_t row0;            // first destination row (transposed: column) of output row m = 0
  const float* gain;       // fp32 [dim] multiplied in before the rotation, or null
  float* ssq;              // fp32 [ssq_np][ssq_stride]: element (t, m) = sum of squares of row m's (acc + bias) over
                           // the t-th run of dim / ssq_np columns of the section (one run per block tile), or null
  int rope;                // rotate channel pairs (2i, 2i+1) of each head by the row's entries of HeadsArgs::cs
  int transposed;          // written channel-major; such tiles are computed with the operands exchanged
};
struct HeadsArgs {
  HeadSection sec[3];
  int dim, head_dim;       // section width, head width
  int64_t ssq_stride;      // >= M
  int ssq_np;              // out: partial sums per row and section that the chosen tile shape produces
  const float2* cs;        // [M][head_dim / 2] (cos, sin) of output row m and channel pair i, for sections with rope
};

struct EpiArgs {
  void* out;            // EPI_STORE / EPI_GELU: [M, ldo] of the activation type; EPI_RESID (bf16 GEMM): optional
                        // copy of the updated residual rows, rounded to bf16 (null = none)
  int64_t ldo;
  const void* bias;     // [N] of the weight type, may be null
  float* resid;         // EPI_RESID: fp32 [M, ldr], updated in place: resid += gate * (acc + bias)
  int64_t ldr;
  const float* gate;    // EPI_RESID: fp32 [N] or null (= 1)
  HeadsArgs* heads;        // EPI_HEADS: host pointer, copied into the launch; its ssq_np is filled in
};
