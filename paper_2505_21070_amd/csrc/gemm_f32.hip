// fp32 GEMM for the DP_F32 path: C = A[M,K] * W[K,N] with a fused epilogue.  Plain FMA arithmetic
// (no matrix cores) so that results stay within fp32 rounding of the reference.
// 64x64 tile per 256-thread block, 4x4 outputs per thread, K stepped by 16 through LDS, the next step's
// operands prefetched into registers.
#include "kernels.h"

template <int EPI>
__global__ __launch_bounds__(256) void k_gemm_f32(const float* __restrict__ A, int64_t lda,
                                                  const float* __restrict__ W, int64_t ldw, int64_t M,
                                                  int64_t N, int64_t K, EpiArgs e) {
  __shared__ float As[16][64 + 4];   // [k][m]
  __shared__ float Ws[16][64 + 4];   // [k][n]
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;        // thread owns rows ty*4.., cols tx*4..
  const int64_t m0 = (int64_t)blockIdx.x * 64, n0 = (int64_t)blockIdx.y * 64;   // rows on x: no 65535-block limit
  float acc[4][4] = {};
  // the next k-step's operands travel from global memory into registers while this one is multiplied
  float ra[4], rw[4];
  auto fetch = [&](int64_t k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {                // A tile: 64 rows x 16 k; W tile: 16 k x 64 columns
      const int idx = tid + i * 256;             // 0..1023
      const int64_t m = m0 + (idx >> 4), ka = k0 + (idx & 15);
      ra[i] = (m < M && ka < K) ? A[m * lda + ka] : 0.f;
      const int64_t kw = k0 + (idx >> 6), n = n0 + (idx & 63);
      rw[i] = (kw < K && n < N) ? W[kw * ldw + n] : 0.f;
    }
  };
  fetch(0);
  for (int64_t k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + i * 256;
      As[idx & 15][idx >> 4] = ra[i];
      Ws[idx >> 6][idx & 63] = rw[i];
    }
    __syncthreads();
    if (k0 + 16 < K) fetch(k0 + 16);
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Ws[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  const float* bias = (const float*)e.bias;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float v = acc[i][j] + (bias ? bias[n] : 0.f);
      if (EPI == EPI_GELU) v = gelu_tanh_f(v);
      if (EPI == EPI_RESID) {
        float* r = e.resid + m * e.ldr + n;
        *r = *r + (e.gate ? e.gate[n] : 1.f) * v;
      } else {
        ((float*)e.out)[m * e.ldo + n] = v;
      }
    }
  }
}

void launch_gemm_f32(const float* A, int64_t lda, const float* W, int64_t ldw, int64_t M, int64_t N,
                     int64_t K, int epi, const EpiArgs& e, hipStream_t st) {
  if (M <= 0 || N <= 0) return;
  dim3 grid((unsigned)((M + 63) / 64), (unsigned)((N + 63) / 64));     // N <= 6 * 8192, so grid.y stays small
  if (epi == EPI_STORE) k_gemm_f32<EPI_STORE><<<grid, 256, 0, st>>>(A, lda, W, ldw, M, N, K, e);
  else if (epi == EPI_GELU) k_gemm_f32<EPI_GELU><<<grid, 256, 0, st>>>(A, lda, W, ldw, M, N, K, e);
  else k_gemm_f32<EPI_RESID><<<grid, 256, 0, st>>>(A, lda, W, ldw, M, N, K, e);
}
