// Measurement aid: the rate at which this GPU issues v_mfma_f32_32x32x16_bf16 when nothing else
// happens (no memory traffic, independent accumulators, two wavefronts per SIMD), for a chosen operand
// bit pattern.  The matrix cores' clock under load depends on how many operand bits toggle, so the
// attainable ceiling for real data lies below the one for zeros; a roofline fraction against the
// published peak is better read next to this figure.
#include <hip/hip_runtime.h>

#include "../../include/dualparal.h"
#include "kernels.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}
// two bf16 values with random sign and mantissa and an exponent of 2^-2 or 2^-1
__device__ __forceinline__ uint32_t random_pair(uint32_t r) {
  const uint32_t lo = (r & 0x80ffu) | (0x3e80u + ((r >> 8) & 0x100u));
  const uint32_t hi = ((r >> 16) & 0x80ffu) | (0x3e80u + ((r >> 24) & 0x100u));
  return lo | (hi << 16);
}

__global__ __launch_bounds__(256) void k_probe_mfma(float* __restrict__ out, int iters, int mode) {
  u32x4 ua, ub;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t ra = mix32(threadIdx.x * 8 + i + blockIdx.x * 7919u);
    const uint32_t rb = mix32(threadIdx.x * 8 + i + 4 + blockIdx.x * 104729u);
    ua[i] = mode == DP_PROBE_ZEROS ? 0u : random_pair(ra);
    ub[i] = mode == DP_PROBE_ZEROS ? 0u : random_pair(rb);
  }
  const bf16x8 a = __builtin_bit_cast(bf16x8, ua), b = __builtin_bit_cast(bf16x8, ub);
  f32x16 acc[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int n = 0; n < 4; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[n], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[n][r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

int dp_set_error(int code, const char* msg);   // defined next to dp_last_error

extern "C" int dp_probe_mfma_bf16(int32_t operand_mode, int32_t iters, float* scratch, int64_t scratch_floats,
                                  void* hip_stream, double* tflops) {
  constexpr int kBlocks = 512;                       // 2 blocks of 4 wavefronts per compute unit
  if (!scratch || !tflops || iters < 1 || scratch_floats < (int64_t)kBlocks * 256 ||
      (operand_mode != DP_PROBE_ZEROS && operand_mode != DP_PROBE_RANDOM)) {
    return dp_set_error(DP_EINVAL, "dp_probe_mfma_bf16: bad argument");
  }
  hipStream_t st = (hipStream_t)hip_stream;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
    return dp_set_error(DP_EHIP, "dp_probe_mfma_bf16: hipEventCreate failed");
  }
  k_probe_mfma<<<kBlocks, 256, 0, st>>>(scratch, iters / 16 + 1, operand_mode);      // warm-up
  (void)hipEventRecord(e0, st);
  k_probe_mfma<<<kBlocks, 256, 0, st>>>(scratch, iters, operand_mode);
  (void)hipEventRecord(e1, st);
  const hipError_t err = hipEventSynchronize(e1);
  float ms = 0.f;
  if (err == hipSuccess) (void)hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (err != hipSuccess || !(ms > 0.f)) {
    return dp_set_error(DP_EHIP, "dp_probe_mfma_bf16: the timed launch failed");
  }
  // blocks x 4 wavefronts x 4 accumulators x iters MFMAs of 2*32*32*16 flops
  *tflops = (double)kBlocks * 4 * 4 * (double)iters * 32768.0 / ((double)ms * 1e9);
  return DP_OK;
}

// A plain streaming pass of the LayerNorm's traffic shape (4 bytes read, 2 bytes written per element, nothing
// else): the library's own fp32 -> bf16 conversion kernel, event-timed.  What it reaches on a buffer of the same
// size is the ceiling any kernel that must read the fp32 residual stream and write bf16 can be held against.
extern "C" int dp_probe_stream_f32_bf16(const float* src, void* dst, int64_t n, int32_t iters, void* hip_stream,
                                        double* gbytes_per_s) {
  if (!src || !dst || !gbytes_per_s || n < 8 || n % 8 || iters < 1 || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15))
    return dp_set_error(DP_EINVAL, "dp_probe_stream_f32_bf16: bad argument");
  hipStream_t st = (hipStream_t)hip_stream;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
    return dp_set_error(DP_EHIP, "dp_probe_stream_f32_bf16: hipEventCreate failed");
  launch_from_f32<bf16_t>(src, (bf16_t*)dst, n, st);                                   // warm-up
  (void)hipEventRecord(e0, st);
  for (int i = 0; i < iters; ++i) launch_from_f32<bf16_t>(src, (bf16_t*)dst, n, st);
  (void)hipEventRecord(e1, st);
  const hipError_t err = hipEventSynchronize(e1);
  float ms = 0.f;
  if (err == hipSuccess) (void)hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (err != hipSuccess || !(ms > 0.f)) return dp_set_error(DP_EHIP, "dp_probe_stream_f32_bf16: the timed launches failed");
  *gbytes_per_s = (double)n * 6.0 * iters / ((double)ms * 1e6);
  return DP_OK;
}
