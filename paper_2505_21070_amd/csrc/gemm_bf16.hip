// bf16 GEMM on the gfx950 matrix cores: C[M,N] = A[M,K] * Wt[N,K]^T, fp32 accumulate, fused epilogue.
// Both operands are K-contiguous, so every MFMA operand fragment is one 16-byte LDS read.
//
// Block tile BM x BN x 64, WGM x WGN wavefronts, each owning a (BM/WGM) x (BN/WGN) sub-tile built from
// v_mfma_f32_32x32x16_bf16.  Global -> registers -> LDS staging with two LDS buffers: the loads of
// k-tile i+1 are in flight while k-tile i is multiplied.  LDS rows are 128 bytes (64 bf16); the
// 16-byte chunk index is XOR-swizzled with (row >> 1) & 7: LDS serves 16 lanes x 16 bytes per cycle from
// 64 banks, i.e. two 128-byte rows per bank sweep, and the swizzle spreads a column of chunks over all of them.
#include "kernels.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int BM, int BN, int WGM, int WGN, int EPI>
__global__ __launch_bounds__(WGM * WGN * 64) void k_gemm_bf16(const bf16_t* __restrict__ A, int64_t lda,
                                                             const bf16_t* __restrict__ Bt, int64_t ldb,
                                                             int64_t M, int64_t N, int64_t K, int tiles_n,
                                                             EpiArgs e) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int CA = BM * 8 / NT, CB = BN * 8 / NT;      // 16-byte chunks per thread per k-tile
  constexpr int STAGE = (BM + BN) * 8;                   // chunks per LDS buffer
  static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/thread mismatch");
  extern __shared__ uint4 smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  // tiles of one XCD (blocks are dealt round-robin over 8 XCDs) form a contiguous run of tile ids
  const int nblk = gridDim.x;
  int pid = blockIdx.x;
  if (nblk % 8 == 0) pid = (pid & 7) * (nblk >> 3) + (pid >> 3);
  const int64_t m0 = (int64_t)(pid / tiles_n) * BM, n0 = (int64_t)(pid % tiles_n) * BN;

  const uint4* ga[CA]; const uint4* gb[CB];
  int sa[CA], sb[CB];
#pragma unroll
  for (int i = 0; i < CA; ++i) {
    const int c = tid + i * NT, row = c >> 3, kc = c & 7;
    ga[i] = (const uint4*)(A + (m0 + row) * lda + kc * 8);
    sa[i] = row * 8 + (kc ^ ((row >> 1) & 7));
  }
#pragma unroll
  for (int i = 0; i < CB; ++i) {
    const int c = tid + i * NT, row = c >> 3, kc = c & 7;
    gb[i] = (const uint4*)(Bt + (n0 + row) * ldb + kc * 8);
    sb[i] = BM * 8 + row * 8 + (kc ^ ((row >> 1) & 7));
  }
  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  uint4 ra[CA], rb[CB];
  const int KT = (int)(K / 64);
#pragma unroll
  for (int i = 0; i < CA; ++i) ra[i] = ga[i][0];
#pragma unroll
  for (int i = 0; i < CB; ++i) rb[i] = gb[i][0];
#pragma unroll
  for (int i = 0; i < CA; ++i) smem[sa[i]] = ra[i];
#pragma unroll
  for (int i = 0; i < CB; ++i) smem[sb[i]] = rb[i];
  __syncthreads();

  const int lr = lane & 31, lg = lane >> 5;
  for (int kt = 0; kt < KT; ++kt) {
    // prefetch the next k-tile (the last iteration re-reads its own tile; the copy is never used)
    const int ktn = kt + 1 < KT ? kt + 1 : kt;
#pragma unroll
    for (int i = 0; i < CA; ++i) ra[i] = ga[i][ktn * 8];            // 8 chunks = 64 bf16 along K
#pragma unroll
    for (int i = 0; i < CB; ++i) rb[i] = gb[i][ktn * 8];
    const uint4* buf = smem + (kt & 1) * STAGE;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 af[TM], bfr[TN];
      const int kc = ks * 2 + lg;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = wm * WM + i * 32 + lr;
        af[i] = __builtin_bit_cast(bf16x8, buf[row * 8 + (kc ^ ((row >> 1) & 7))]);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int row = wn * WN + j * 32 + lr;
        bfr[j] = __builtin_bit_cast(bf16x8, buf[BM * 8 + row * 8 + (kc ^ ((row >> 1) & 7))]);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    {
      uint4* nb = smem + ((kt + 1) & 1) * STAGE;
#pragma unroll
      for (int i = 0; i < CA; ++i) nb[sa[i]] = ra[i];
#pragma unroll
      for (int i = 0; i < CB; ++i) nb[sb[i]] = rb[i];
    }
    __syncthreads();
  }

  // epilogue: lane holds column n = .. + lr and rows (r/4)*8 + lg*4 + (r%4) of every 32x32 tile
  const bf16_t* bias = (const bf16_t*)e.bias;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int64_t n = n0 + wn * WN + j * 32 + lr;
    if (n >= N) continue;
    const float bv = bias ? bf16_to_f32(bias[n]) : 0.f;
    float gv = 1.f;
    if (EPI == EPI_RESID && e.gate) gv = e.gate[n];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t m = m0 + wm * WM + i * 32 + (r >> 2) * 8 + lg * 4 + (r & 3);
        if (m >= M) continue;
        float v = acc[i][j][r] + bv;
        if (EPI == EPI_GELU) v = gelu_tanh_f(v);
        if (EPI == EPI_RESID) {
          float* p = e.resid + m * e.ldr + n;
          *p = *p + gv * v;
        } else {
          ((bf16_t*)e.out)[m * e.ldo + n] = f32_to_bf16(v);
        }
      }
    }
  }
}

template <int BM, int BN, int WGM, int WGN>
static void launch_cfg(const bf16_t* A, int64_t lda, const bf16_t* Wt, int64_t ldw, int64_t M, int64_t N,
                       int64_t K, int epi, const EpiArgs& e, hipStream_t st) {
  constexpr int NT = WGM * WGN * 64;
  constexpr size_t lds = (size_t)(BM + BN) * 128 * 2;
  const int tm = (int)((M + BM - 1) / BM), tn = (int)((N + BN - 1) / BN);
  static bool attr_done = false;
  if (!attr_done) {
    (void)hipFuncSetAttribute((const void*)k_gemm_bf16<BM, BN, WGM, WGN, EPI_STORE>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    (void)hipFuncSetAttribute((const void*)k_gemm_bf16<BM, BN, WGM, WGN, EPI_GELU>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    (void)hipFuncSetAttribute((const void*)k_gemm_bf16<BM, BN, WGM, WGN, EPI_RESID>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attr_done = true;
  }
  dim3 grid((unsigned)(tm * tn));
  if (epi == EPI_STORE) k_gemm_bf16<BM, BN, WGM, WGN, EPI_STORE><<<grid, NT, lds, st>>>(A, lda, Wt, ldw, M, N, K, tn, e);
  else if (epi == EPI_GELU) k_gemm_bf16<BM, BN, WGM, WGN, EPI_GELU><<<grid, NT, lds, st>>>(A, lda, Wt, ldw, M, N, K, tn, e);
  else k_gemm_bf16<BM, BN, WGM, WGN, EPI_RESID><<<grid, NT, lds, st>>>(A, lda, Wt, ldw, M, N, K, tn, e);
}

void launch_gemm_bf16(const bf16_t* A, int64_t lda, const bf16_t* Wt, int64_t ldw, int64_t M, int64_t N,
                      int64_t K, int epi, const EpiArgs& e, hipStream_t st) {
  if (M <= 0 || N <= 0) return;
  // small problems: 128x128 tiles keep more CUs busy; large ones: 256x256 for operand reuse
  const int64_t big_tiles = ((M + 255) / 256) * ((N + 255) / 256);
  if (big_tiles >= 256) launch_cfg<256, 256, 2, 4>(A, lda, Wt, ldw, M, N, K, epi, e, st);
  else launch_cfg<128, 128, 2, 2>(A, lda, Wt, ldw, M, N, K, epi, e, st);
}
