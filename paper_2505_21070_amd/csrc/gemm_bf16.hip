// bf16 GEMM on the gfx950 matrix cores: C[M,N] = A[M,K] * Wt[N,K]^T, fp32 accumulate, fused epilogue.
// Both operands are K-contiguous, so every MFMA operand fragment is one 16-byte LDS read.
//
// Block tile BM x BN x 64, WGM x WGN wavefronts, each owning a (BM/WGM) x (BN/WGN) sub-tile built from
// v_mfma_f32_32x32x16_bf16.  k-tiles go HBM -> LDS directly (no staging registers, no LDS stores): the
// loads of k-tile kt+1 are issued before k-tile kt is multiplied and are waited for at the barrier that
// ends the iteration.  Operand fragments are double-buffered in registers: those of k-step ks+1 are
// read from LDS while the MFMAs of k-step ks run.  LDS rows are 128 bytes (64 bf16); LDS serves 16 lanes
// x 16 bytes per cycle from 64 banks, i.e. two rows per bank sweep, so the 16-byte chunk index is
// XOR-swizzled with (row >> 1) & 7, which spreads a column of chunks over all banks.
//
// Split-K (residual epilogue only): the k-tiles are divided among `splits` blocks per output tile which
// add their partial products into the fp32 residual stream with hardware float atomics, so that small-N
// GEMMs still fill the 256 CUs.
#include "kernels.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void glb_void_t;

// tanh-GELU through the logistic function: 0.5 x (1 + tanh(u)) = x / (1 + exp(-2u))
__device__ __forceinline__ float gelu_tanh_fast(float v) {
  const float u2 = -2.0f * 0.7978845608028654f * 1.4426950408889634f * (v + 0.044715f * v * v * v);   // -2u log2(e)
  return v * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(u2));
}

template <int BM, int BN, int WGM, int WGN, int EPI>
__global__ __launch_bounds__(WGM * WGN * 64) void k_gemm_bf16(const bf16_t* __restrict__ A, int64_t lda,
                                                             const bf16_t* __restrict__ Bt, int64_t ldb,
                                                             int64_t M, int64_t N, int64_t K, int tiles_n,
                                                             int tiles, int splits, EpiArgs e) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int IA = BM * 8 / NT, IB = BN * 8 / NT;      // wavefront load instructions per k-tile (64 chunks each)
  constexpr int STAGE = (BM + BN) * 8;                   // 16-byte chunks per LDS buffer
  static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/thread mismatch");
  extern __shared__ uint4 smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  // Blocks are dealt round-robin over the 8 XCDs, each with its own L2: give every XCD a contiguous run
  // of work ids (row-major tiles, so neighbours share the A row-panel and walk the B panels together).
  // The grid is padded to a multiple of 8; the padding blocks have nothing to do.
  const int pid = (int)(blockIdx.x & 7) * (int)(gridDim.x >> 3) + (int)(blockIdx.x >> 3);
  if (pid >= tiles * splits) return;
  const int split = pid / tiles, tile = pid % tiles;
  // tiles are walked in bands of 4 tile rows, column by column inside a band: the ~32 blocks an XCD runs
  // at a time then cover about 4 x 8 tiles and share 4 A panels and 8 B panels instead of 1 and 32
  const int tiles_m = tiles / tiles_n;
  const int band = tile / (4 * tiles_n), in_band = tile % (4 * tiles_n);
  const int band_rows = tiles_m - band * 4 < 4 ? tiles_m - band * 4 : 4;
  const int64_t m0 = (int64_t)(band * 4 + in_band % band_rows) * BM, n0 = (int64_t)(in_band / band_rows) * BN;
  const int KT_all = (int)(K / 64);
  const int kt0 = (int)((int64_t)KT_all * split / splits), KT = (int)((int64_t)KT_all * (split + 1) / splits) - kt0;

  // slot p of a tile holds chunk (p & 7) ^ ((row >> 1) & 7) of row p >> 3; one wavefront instruction
  // fills slots [base, base + 64), lane l the slot base + l
  const bf16_t* gA[IA]; const bf16_t* gB[IB];
#pragma unroll
  for (int i = 0; i < IA; ++i) {
    const int p = (wave * IA + i) * 64 + lane, row = p >> 3, ch = (p & 7) ^ ((row >> 1) & 7);
    gA[i] = A + (m0 + row) * lda + (int64_t)kt0 * 64 + ch * 8;
  }
#pragma unroll
  for (int i = 0; i < IB; ++i) {
    const int p = (wave * IB + i) * 64 + lane, row = p >> 3, ch = (p & 7) ^ ((row >> 1) & 7);
    gB[i] = Bt + (n0 + row) * ldb + (int64_t)kt0 * 64 + ch * 8;
  }
  auto load_tile = [&](int kt, int bufi) __attribute__((always_inline)) {
    const int t = (kt < KT ? kt : KT - 1) * 64;            // past the end: the last tile again, never used
    uint4* base = smem + bufi * STAGE;
#pragma unroll
    for (int i = 0; i < IA; ++i)
      __builtin_amdgcn_global_load_lds((glb_void_t*)(gA[i] + t), (lds_void_t*)(base + (wave * IA + i) * 64), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < IB; ++i)
      __builtin_amdgcn_global_load_lds((glb_void_t*)(gB[i] + t), (lds_void_t*)(base + BM * 8 + (wave * IB + i) * 64), 16, 0, 0);
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int lr = lane & 31, lg = lane >> 5;
  int arow[TM], brow[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) arow[i] = wm * WM + i * 32 + lr;
#pragma unroll
  for (int j = 0; j < TN; ++j) brow[j] = wn * WN + j * 32 + lr;

  load_tile(0, 0);
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    load_tile(kt + 1, (kt + 1) & 1);
    const uint4* buf = smem + (kt & 1) * STAGE;
    bf16x8 af[2][TM], bfr[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) af[0][i] = __builtin_bit_cast(bf16x8, buf[arow[i] * 8 + (lg ^ ((arow[i] >> 1) & 7))]);
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[0][j] = __builtin_bit_cast(bf16x8, buf[BM * 8 + brow[j] * 8 + (lg ^ ((brow[j] >> 1) & 7))]);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      if (ks < 3) {
        const int kc = (ks + 1) * 2 + lg;
#pragma unroll
        for (int i = 0; i < TM; ++i) af[(ks + 1) & 1][i] = __builtin_bit_cast(bf16x8, buf[arow[i] * 8 + (kc ^ ((arow[i] >> 1) & 7))]);
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[(ks + 1) & 1][j] = __builtin_bit_cast(bf16x8, buf[BM * 8 + brow[j] * 8 + (kc ^ ((brow[j] >> 1) & 7))]);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][i], bfr[ks & 1][j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();      // the next k-tile has landed and every wavefront is done with this one
  }

  // epilogue: lane holds column n = .. + lr and rows (r/4)*8 + lg*4 + (r%4) of every 32x32 tile
  const bf16_t* bias = (const bf16_t*)e.bias;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int64_t n = n0 + wn * WN + j * 32 + lr;
    if (n >= N) continue;
    const float bv = (bias && split == 0) ? bf16_to_f32(bias[n]) : 0.f;
    float gv = 1.f;
    if (EPI == EPI_RESID && e.gate) gv = e.gate[n];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t m = m0 + wm * WM + i * 32 + (r >> 2) * 8 + lg * 4 + (r & 3);
        if (m >= M) continue;
        float v = acc[i][j][r] + bv;
        if (EPI == EPI_GELU) v = gelu_tanh_fast(v);
        if (EPI == EPI_RESID) {
          float* p = e.resid + m * e.ldr + n;
          if (splits > 1) unsafeAtomicAdd(p, gv * v); else *p = *p + gv * v;
        } else {
          ((bf16_t*)e.out)[m * e.ldo + n] = f32_to_bf16(v);
        }
      }
    }
  }
}

template <int BM, int BN, int WGM, int WGN>
static void launch_cfg(const bf16_t* A, int64_t lda, const bf16_t* Wt, int64_t ldw, int64_t M, int64_t N,
                       int64_t K, int epi, int splits, const EpiArgs& e, hipStream_t st) {
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
  dim3 grid((unsigned)((tm * tn * splits + 7) / 8 * 8));
  if (epi == EPI_STORE) k_gemm_bf16<BM, BN, WGM, WGN, EPI_STORE><<<grid, NT, lds, st>>>(A, lda, Wt, ldw, M, N, K, tn, tm * tn, splits, e);
  else if (epi == EPI_GELU) k_gemm_bf16<BM, BN, WGM, WGN, EPI_GELU><<<grid, NT, lds, st>>>(A, lda, Wt, ldw, M, N, K, tn, tm * tn, splits, e);
  else k_gemm_bf16<BM, BN, WGM, WGN, EPI_RESID><<<grid, NT, lds, st>>>(A, lda, Wt, ldw, M, N, K, tn, tm * tn, splits, e);
}

static double cu_fill(int64_t blocks) { return (double)blocks / (double)(((blocks + 255) / 256) * 256); }

void launch_gemm_bf16(const bf16_t* A, int64_t lda, const bf16_t* Wt, int64_t ldw, int64_t M, int64_t N,
                      int64_t K, int epi, const EpiArgs& e, hipStream_t st) {
  if (M <= 0 || N <= 0) return;
  // One block per CU at a time, so a launch costs ceil(blocks / 256) rounds of one block's duration.
  // 256x256 tiles have the most operand reuse; 192x256 tiles trade a little of it for more blocks when
  // that fills the last round better; tiny problems take 128x128 tiles.
  const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256);
  const int64_t t192 = ((M + 191) / 192) * ((N + 255) / 256);
  if (t256 < 64) { launch_cfg<128, 128, 2, 2>(A, lda, Wt, ldw, M, N, K, epi, 1, e, st); return; }
  const double cost256 = (double)((t256 + 255) / 256), cost192 = 0.78 * (double)((t192 + 255) / 256);
  (void)cu_fill;
  if (cost192 < cost256) launch_cfg<192, 256, 2, 4>(A, lda, Wt, ldw, M, N, K, epi, 1, e, st);
  else launch_cfg<256, 256, 2, 4>(A, lda, Wt, ldw, M, N, K, epi, 1, e, st);
}
