// bf16 GEMM on the gfx950 matrix cores: C[M,N] = A[M,K] * Wt[N,K]^T, fp32 accumulate, fused epilogue.
// Both operands are K-contiguous, so every MFMA operand fragment is one 16-byte LDS read.
//
// Block tile BM x BN x 64, WGM x WGN wavefronts, each owning a (BM/WGM) x (BN/WGN) sub-tile built from
// v_mfma_f32_32x32x16_bf16.  k-tiles go HBM -> LDS directly (no staging registers, no LDS stores) into
// two buffers: k-tile kt+1 is in flight while k-tile kt is multiplied.  Operand fragments are
// double-buffered in registers: those of k-step ks+1 are read from LDS while the MFMAs of k-step ks run.  LDS rows are 128 bytes (64 bf16); LDS serves 16 lanes
// x 16 bytes per cycle from 64 banks, i.e. two rows per bank sweep, so the 16-byte chunk index is
// XOR-swizzled with (row >> 1) & 7, which spreads a column of chunks over all banks.
//
// The epilogue stages the output tile through LDS so that global memory is written (and, for the fp32
// residual update, read) in whole rows, 16 bytes per lane.
#include "kernels.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void glb_void_t;

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t cvt_pk_bf16(float a, float b) {
  f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// tanh-GELU through the logistic function: 0.5 x (1 + tanh(u)) = x / (1 + exp(-2u))
__device__ __forceinline__ float gelu_tanh_fast(float v) {
  const float u2 = -2.0f * 0.7978845608028654f * 1.4426950408889634f * (v + 0.044715f * v * v * v);   // -2u log2(e)
  return v * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(u2));
}

template <int BM, int BN, int WGM, int WGN, int EPI>
__global__ __launch_bounds__(WGM * WGN * 64) void k_gemm_bf16(const bf16_t* __restrict__ A, int64_t lda,
                                                             const bf16_t* __restrict__ Bt, int64_t ldb,
                                                             int64_t M, int64_t N, int64_t K, int tiles_n,
                                                             int tiles, EpiArgs e) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int IA = (BM * 8 + NT - 1) / NT, IB = BN * 8 / NT;   // wavefront load instructions per k-tile (64 chunks each)
  constexpr bool A_RAGGED = BM * 8 % NT != 0;                  // the last wavefronts' share of the A tile is shorter
  constexpr int STAGE = (BM + BN) * 8;                   // 16-byte chunks per LDS buffer
  static_assert(BM * 8 % 64 == 0 && BN * 8 % NT == 0, "tile/thread mismatch");
  extern __shared__ uint4 smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  // Blocks are dealt round-robin over the 8 XCDs, each with its own L2: give every XCD a contiguous run
  // of work ids (row-major tiles, so neighbours share the A row-panel and walk the B panels together).
  // The grid is padded to a multiple of 8; the padding blocks have nothing to do.
  const int pid = (int)(blockIdx.x & 7) * (int)(gridDim.x >> 3) + (int)(blockIdx.x >> 3);
  if (pid >= tiles) return;
  const int tile = pid;
  // tiles are walked in bands of 4 tile rows, column by column inside a band: the ~32 blocks an XCD runs
  // at a time then cover about 4 x 8 tiles and share 4 A panels and 8 B panels instead of 1 and 32
  const int tiles_m = tiles / tiles_n;
  const int band = tile / (4 * tiles_n), in_band = tile % (4 * tiles_n);
  const int band_rows = tiles_m - band * 4 < 4 ? tiles_m - band * 4 : 4;
  const int64_t m0 = (int64_t)(band * 4 + in_band % band_rows) * BM, n0 = (int64_t)(in_band / band_rows) * BN;
  const int KT = (int)(K / 64);

  // slot p of a tile holds chunk (p & 7) ^ ((row >> 1) & 7) of row p >> 3; one wavefront instruction
  // fills slots [base, base + 64), lane l the slot base + l
  const bf16_t* gA[IA]; const bf16_t* gB[IB];
#pragma unroll
  for (int i = 0; i < IA; ++i) {
    const int p = (wave * IA + i) * 64 + lane, row = p >> 3, ch = (p & 7) ^ ((row >> 1) & 7);
    gA[i] = A + (m0 + row) * lda + ch * 8;
  }
#pragma unroll
  for (int i = 0; i < IB; ++i) {
    const int p = (wave * IB + i) * 64 + lane, row = p >> 3, ch = (p & 7) ^ ((row >> 1) & 7);
    gB[i] = Bt + (n0 + row) * ldb + ch * 8;
  }
  auto load_tile = [&](int kt, int bufi) __attribute__((always_inline)) {
    if (kt >= KT) return;
    const int t = kt * 64;
    uint4* base = smem + bufi * STAGE;
#pragma unroll
    for (int i = 0; i < IA; ++i)
      if (!A_RAGGED || (wave * IA + i) * 64 < BM * 8)
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

  // Software pipeline.  k-tile kt+1 is in flight while k-tile kt is multiplied; the fragments of k-step
  // ks+1 are read while the MFMAs of k-step ks run.  The barrier of an iteration sits before its last
  // k-step, whose fragments are already in registers: behind it the buffer of k-tile kt is free for
  // k-tile kt+2 and k-tile kt+1 has landed, so the first fragments of the next iteration are read there.
  auto read_frags = [&](const uint4* buf, int ks, bf16x8* af, bf16x8* bfr) __attribute__((always_inline)) {
    const int kc = ks * 2 + lg;
#pragma unroll
    for (int i = 0; i < TM; ++i) af[i] = __builtin_bit_cast(bf16x8, buf[arow[i] * 8 + (kc ^ ((arow[i] >> 1) & 7))]);
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[j] = __builtin_bit_cast(bf16x8, buf[BM * 8 + brow[j] * 8 + (kc ^ ((brow[j] >> 1) & 7))]);
  };
  bf16x8 af[2][TM], bfr[2][TN];
  load_tile(0, 0);
  tile_barrier();
  load_tile(1, 1);
  read_frags(smem, 0, af[0], bfr[0]);
  for (int kt = 0; kt < KT; ++kt) {
    const uint4* buf = smem + (kt & 1) * STAGE;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      if (ks < 3) {
        read_frags(buf, ks + 1, af[(ks + 1) & 1], bfr[(ks + 1) & 1]);
      } else {
        tile_barrier();
        load_tile(kt + 2, kt & 1);
        read_frags(smem + ((kt + 1) & 1) * STAGE, 0, af[0], bfr[0]);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ks & 1][j], af[ks & 1][i], acc[i][j], 0, 0, 0);
      // issue order: the LDS reads (and, in the last k-step, the k-tile loads) are spread between the MFMAs
      if (ks < 3) {
#pragma unroll
        for (int g = 0; g < TM + TN; ++g) {
          __builtin_amdgcn_sched_group_barrier(0x008, (TM * TN) / (TM + TN), 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - (TM + TN) * ((TM * TN) / (TM + TN)), 0);
      }
      __builtin_amdgcn_sched_barrier(0);      // nothing moves between k-steps: reads stay one step ahead
    }
  }

  // Epilogue.  The MFMAs ran with the weight rows as the A operand, so a lane holds the output row
  // m = .. + lr and, per register quad q, the four consecutive columns n = .. + q*8 + lg*4 + (0..3).
  // The tile goes through LDS (free now) so that global memory sees whole rows: 16 bytes per lane,
  // consecutive lanes on consecutive addresses.  LDS rows are XOR-swizzled with the row index so that
  // neither the column-wise writes nor the row-wise reads conflict on banks.
  constexpr int NW = WGM * WGN;
  const bf16_t* bias = (const bf16_t*)e.bias;
  if constexpr (EPI != EPI_RESID) {
    constexpr int UPR = BN / 4;                          // 8-byte units (4 bf16) per LDS row
    constexpr int CPR = BN / 8, RPI = 64 / CPR;          // 16-byte chunks per row, rows per wavefront read
    // the whole tile at once if it fits the two operand buffers, else one wavefront row (WM rows) per pass
    constexpr int SP = (BM * BN * 2 <= (BM + BN) * 256) ? 1 : WGM, RP = BM / SP;
    uint2* l8 = (uint2*)smem;
#pragma unroll
    for (int pass = 0; pass < SP; ++pass) {
      __syncthreads();                                   // the operand tiles / the previous pass are done with
      if (SP == 1 || wm == pass) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int nl = wn * WN + j * 32 + q * 8 + lg * 4;
            float bv[4] = {0.f, 0.f, 0.f, 0.f};
            if (bias && n0 + nl < N) {
              const uint2 b4 = *(const uint2*)(bias + n0 + nl);
              bv[0] = bf16_to_f32((bf16_t)(b4.x & 0xffff)); bv[1] = bf16_to_f32((bf16_t)(b4.x >> 16));
              bv[2] = bf16_to_f32((bf16_t)(b4.y & 0xffff)); bv[3] = bf16_to_f32((bf16_t)(b4.y >> 16));
            }
#pragma unroll
            for (int i = 0; i < TM; ++i) {
              const int row = (SP == 1 ? wm * WM : 0) + i * 32 + lr;      // row inside this pass
              float v[4];
#pragma unroll
              for (int t = 0; t < 4; ++t) {
                v[t] = acc[i][j][q * 4 + t] + bv[t];
                if (EPI == EPI_GELU) v[t] = gelu_tanh_fast(v[t]);
              }
              uint2 pk;
              pk.x = cvt_pk_bf16(v[0], v[1]);
              pk.y = cvt_pk_bf16(v[2], v[3]);
              l8[row * UPR + ((nl >> 2) ^ (row & 31))] = pk;
            }
          }
      }
      __syncthreads();
#pragma unroll
      for (int it = 0; it < RP / NW / RPI; ++it) {
        const int row = wave * (RP / NW) + it * RPI + lane / CPR, p = lane % CPR;
        uint4 d = smem[row * CPR + p];
        // the chunk read holds units 2p and 2p+1 of the swizzled row, i.e. the two halves of logical
        // chunk p ^ ((row & 31) >> 1), exchanged when the row index is odd
        if (row & 1) d = make_uint4(d.z, d.w, d.x, d.y);
        const int64_t m = m0 + pass * RP + row, n = n0 + (p ^ ((row & 31) >> 1)) * 8;
        if (m < M && n < N) *(uint4*)((bf16_t*)e.out + m * e.ldo + n) = d;
      }
    }
  } else {
    // residual stream: x[m, n] += gate[n] * (acc + bias[n]) in fp32.  Passes over the wavefront rows of the
    // block tile and, inside one, over groups of GI 32-row accumulator tiles: as many as fit in LDS as floats
    constexpr int CPR = BN / 4, RPI = 64 / CPR;          // 16-byte chunks (4 floats) per row
    constexpr int GI_FIT = (BM + BN) * 256 / (32 * BN * 4), GI = GI_FIT < TM ? GI_FIT : TM;
    static_assert(GI >= 1, "one 32-row tile of fp32 results must fit the operand buffers");
    float4* l16 = (float4*)smem;
#pragma unroll
    for (int pass = 0; pass < WGM; ++pass) {
#pragma unroll
      for (int i0 = 0; i0 < TM; i0 += GI) {
        const int gi = TM - i0 < GI ? TM - i0 : GI;      // accumulator tiles in this group
        __syncthreads();
        if (wm == pass) {
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const int nl = wn * WN + j * 32 + q * 8 + lg * 4;
              float bv[4] = {0.f, 0.f, 0.f, 0.f};
              float4 gv = make_float4(1.f, 1.f, 1.f, 1.f);
              if (n0 + nl < N) {
                if (bias) {
                  const uint2 b4 = *(const uint2*)(bias + n0 + nl);
                  bv[0] = bf16_to_f32((bf16_t)(b4.x & 0xffff)); bv[1] = bf16_to_f32((bf16_t)(b4.x >> 16));
                  bv[2] = bf16_to_f32((bf16_t)(b4.y & 0xffff)); bv[3] = bf16_to_f32((bf16_t)(b4.y >> 16));
                }
                if (e.gate) gv = *(const float4*)(e.gate + n0 + nl);
              }
#pragma unroll
              for (int ii = 0; ii < GI; ++ii) {
                if (i0 + ii < TM) {
                  const int row = ii * 32 + lr;
                  float4 v;
                  v.x = gv.x * (acc[i0 + ii][j][q * 4 + 0] + bv[0]);
                  v.y = gv.y * (acc[i0 + ii][j][q * 4 + 1] + bv[1]);
                  v.z = gv.z * (acc[i0 + ii][j][q * 4 + 2] + bv[2]);
                  v.w = gv.w * (acc[i0 + ii][j][q * 4 + 3] + bv[3]);
                  l16[row * CPR + ((nl >> 2) ^ (row & 15))] = v;
                }
              }
            }
        }
        __syncthreads();
        // gi * 32 rows, shared out over the wavefronts RPI rows per read
        for (int r = wave * RPI; r < gi * 32; r += NW * RPI) {
          const int row = r + lane / CPR, p = lane % CPR;
          const float4 v = l16[row * CPR + p];
          const int64_t m = m0 + pass * WM + i0 * 32 + row, n = n0 + (p ^ (row & 15)) * 4;
          if (m < M && n < N) {
            float4* x = (float4*)(e.resid + m * e.ldr + n);
            float4 xv = *x;
            xv.x += v.x; xv.y += v.y; xv.z += v.z; xv.w += v.w;
            *x = xv;
          }
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
  static std::atomic<uint64_t> done[3];
  if (epi == EPI_STORE) allow_dynamic_lds((const void*)k_gemm_bf16<BM, BN, WGM, WGN, EPI_STORE>, (int)lds, done[0]);
  else if (epi == EPI_GELU) allow_dynamic_lds((const void*)k_gemm_bf16<BM, BN, WGM, WGN, EPI_GELU>, (int)lds, done[1]);
  else allow_dynamic_lds((const void*)k_gemm_bf16<BM, BN, WGM, WGN, EPI_RESID>, (int)lds, done[2]);
  dim3 grid((unsigned)((tm * tn + 7) / 8 * 8));
  if (epi == EPI_STORE) k_gemm_bf16<BM, BN, WGM, WGN, EPI_STORE><<<grid, NT, lds, st>>>(A, lda, Wt, ldw, M, N, K, tn, tm * tn, e);
  else if (epi == EPI_GELU) k_gemm_bf16<BM, BN, WGM, WGN, EPI_GELU><<<grid, NT, lds, st>>>(A, lda, Wt, ldw, M, N, K, tn, tm * tn, e);
  else k_gemm_bf16<BM, BN, WGM, WGN, EPI_RESID><<<grid, NT, lds, st>>>(A, lda, Wt, ldw, M, N, K, tn, tm * tn, e);
}

void launch_gemm_bf16(const bf16_t* A, int64_t lda, const bf16_t* Wt, int64_t ldw, int64_t M, int64_t N,
                      int64_t K, int epi, const EpiArgs& e, hipStream_t st) {
  if (M <= 0 || N <= 0) return;
  // One block per CU at a time, so a launch costs ceil(blocks / 256) rounds of one block's duration.
  // 256x256 tiles are the default.  Other shapes are taken when rounds x relative duration comes out lower:
  // 192x256 (0.82 of a 256x256 tile), 160x256 (0.79; 1 x 8 wavefronts, more LDS reads per MFMA, but e.g. 39 x 6
  // tiles fill one round where 33 x 6 leave 58 CUs idle) and 320x256 (1.25, fewer operand bytes per flop).
  // The 160- and 320-row tiles read rows beyond M up to their own multiple, so they are used only where
  // that stays inside the 256-row padding the caller guarantees.  Tiny problems take 128x128 tiles.
  const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256);
  const int64_t t192 = ((M + 191) / 192) * ((N + 255) / 256);
  const int64_t t160 = ((M + 159) / 160) * ((N + 255) / 256);
  const int64_t t320 = ((M + 319) / 320) * ((N + 255) / 256);
  if (t256 < 64) { launch_cfg<128, 128, 2, 2>(A, lda, Wt, ldw, M, N, K, epi, e, st); return; }
  const int64_t mpad = (M + 255) / 256 * 256;
  const double cost256 = (double)((t256 + 255) / 256), cost192 = 0.82 * (double)((t192 + 255) / 256);
  const double cost160 = (M + 159) / 160 * 160 <= mpad ? 0.79 * (double)((t160 + 255) / 256) : 1e30;
  const double cost320 = (M + 319) / 320 * 320 <= mpad ? 1.25 * (double)((t320 + 255) / 256) : 1e30;
  const double best = fmin(fmin(cost256, cost192), fmin(cost160, cost320));
  if (best == cost256) { launch_cfg<256, 256, 2, 4>(A, lda, Wt, ldw, M, N, K, epi, e, st); return; }
  if (best == cost160) { launch_cfg<160, 256, 1, 8>(A, lda, Wt, ldw, M, N, K, epi, e, st); return; }
  if (best == cost320) { launch_cfg<320, 256, 2, 4>(A, lda, Wt, ldw, M, N, K, epi, e, st); return; }
  launch_cfg<192, 256, 2, 4>(A, lda, Wt, ldw, M, N, K, epi, e, st);
}
