// bf16 GEMM on the gfx950 matrix cores: C[M,N] = A[M,K] * Wt[N,K]^T, fp32 accumulate, fused epilogue.
// Both operands are K-contiguous, so every MFMA operand fragment is one 16-byte LDS read.
//
// Block tile BM x BN x 64, WGM x WGN wavefronts, each owning a (BM/WGM) x (BN/WGN) sub-tile built from
// v_mfma_f32_32x32x16_bf16.  k-tiles go HBM -> LDS directly (no staging registers, no LDS stores) into
// two buffers: k-tile kt+1 is in flight while k-tile kt is multiplied.  Operand fragments are
// double-buffered in registers: those of k-step ks+1 are read from LDS while the MFMAs of k-step ks run.
// The issue order of the main loop is pinned (see there): the two wavefronts of a SIMD are served oldest
// first rather than interleaved, so each has to keep the matrix pipe busy on its own; tile loads go out
// one behind an MFMA instead of in a burst, and an MFMA waits only for the LDS reads it needs.
// LDS rows are 128 bytes (64 bf16); LDS serves 16 lanes x 16 bytes per cycle from 64 banks, i.e. two rows per
// bank sweep, so the 16-byte chunk index is XOR-swizzled with (row >> 1) & 7, which spreads a column of
// chunks over all banks.
//
// The epilogue stages the output tile through LDS so that global memory is written (and, for the fp32
// residual update, read) in whole rows, 16 bytes per lane.  EPI_HEADS stores per attention head (q | k | v
// sections: channel gains, 3D rotation, transposed V, row sums of squares for a deferred RMSNorm).
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

// The fragments of a k-step are read in the order A row-tile 0, B column-tiles 0 .. TN-1, A row-tiles 1 ..;
// the MFMAs run row-tile by row-tile (n = i * TN + j).  Index of the last fragment MFMA n needs:
template <int TN> constexpr int frag_need(int n) {
  const int i = n / TN, j = n % TN, ia = i == 0 ? 0 : TN + i, ib = 1 + j;
  return ia > ib ? ia : ib;
}
template <int TN> constexpr int frag_need_upto(int n) {
  int m = -1;
  for (int t = 0; t <= n; ++t) m = frag_need<TN>(t) > m ? frag_need<TN>(t) : m;
  return m;
}
// reads k (issued behind MFMA first + k * (NM - first) / NR) that precede MFMA n
template <int NM, int NR> constexpr int reads_before(int n, int first) {
  int c = 0;
  for (int k = 0; k < NR; ++k) c += first + k * (NM - first) / NR < n ? 1 : 0;
  return c;
}
template <int BM, int BN, int WGM, int WGN, int EPI>
__global__ __launch_bounds__(WGM * WGN * 64) void k_gemm_bf16(const bf16_t* __restrict__ A, int64_t lda,
                                                             const bf16_t* __restrict__ Bt, int64_t ldb,
                                                             int64_t M, int64_t N, int64_t K, int tiles_n,
                                                             int tiles, EpiArgs e, HeadsArgs ha) {
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

  // EPI_HEADS: a tile of a section that is stored channel-major is computed with the operands exchanged
  // (square tiles only), so that its accumulators, staging tile and row stores are those of C^T
  int sec = 0;
  bool swapped = false;
  if constexpr (EPI == EPI_HEADS) {
    sec = (int)(n0 / ha.dim);
    if constexpr (BM == BN) swapped = ha.sec[sec].transposed != 0;
  }
  const bf16_t* const pa = swapped ? Bt + n0 * ldb : A + m0 * lda;
  const bf16_t* const pb = swapped ? A + m0 * lda : Bt + n0 * ldb;
  const int64_t lpa = swapped ? ldb : lda, lpb = swapped ? lda : ldb;
  // slot p of a tile holds chunk (p & 7) ^ ((row >> 1) & 7) of row p >> 3; one wavefront instruction
  // fills slots [base, base + 64), lane l the slot base + l
  const bf16_t* gA[IA]; const bf16_t* gB[IB];
#pragma unroll
  for (int i = 0; i < IA; ++i) {
    const int p = (wave * IA + i) * 64 + lane, row = p >> 3, ch = (p & 7) ^ ((row >> 1) & 7);
    gA[i] = pa + row * lpa + ch * 8;
  }
#pragma unroll
  for (int i = 0; i < IB; ++i) {
    const int p = (wave * IB + i) * 64 + lane, row = p >> 3, ch = (p & 7) ^ ((row >> 1) & 7);
    gB[i] = pb + row * lpb + ch * 8;
  }
  // load instruction q < IA + IB of this wavefront's share of k-tile kt into stage bufi
  auto load_part = [&](int kt, int bufi, int q) __attribute__((always_inline)) {
    if (kt >= KT) return;
    const int t = kt * 64;
    uint4* base = smem + bufi * STAGE;
    if (q < IA) {
      if (!A_RAGGED || (wave * IA + q) * 64 < BM * 8)
        __builtin_amdgcn_global_load_lds((glb_void_t*)(gA[q] + t), (lds_void_t*)(base + (wave * IA + q) * 64), 16, 0, 0);
    } else {
      __builtin_amdgcn_global_load_lds((glb_void_t*)(gB[q - IA] + t), (lds_void_t*)(base + BM * 8 + (wave * IB + q - IA) * 64), 16, 0, 0);
    }
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
  // ks+1 are read while the MFMAs of k-step ks run, one read behind each of the first MFMAs, in the order in
  // which the next step's MFMAs first need them.  The LDS reads are issued through inline assembly and
  // waited for with explicit counts: the compiler would wait for all outstanding reads before the first
  // MFMA of a step (the last of them only two MFMAs old), which stalls a wavefront whenever the other
  // wavefront of its SIMD is not there to fill the gap; here an MFMA waits only for the fragments it
  // needs, issued most of a k-step earlier.  LDS returns reads in order, so "at most c reads outstanding"
  // means every read but the c newest has landed.
  constexpr int NM = TM * TN, NR = TM + TN;              // MFMAs and fragment reads per k-step
  constexpr int NB = NM >= 8 ? 2 : 1;                    // MFMAs of the last k-step issued before the barrier
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_void_t*)smem;
  static_assert(WM % 16 == 0 && WN % 16 == 0, "every fragment row of a lane has the same swizzle");
  // chunk (ks * 2 + lg) ^ s of a row, s = (row >> 1) & 7 = (lr >> 1) & 7 for all of this lane's fragment rows,
  // is at byte (ks * 32) ^ swz of the row
  const uint32_t swz = (uint32_t)(lg ^ ((lr >> 1) & 7)) * 16;
  uint32_t fbase[NR];                                    // fragment f: LDS byte offset of this lane's row in stage 0
#pragma unroll
  for (int f = 0; f < NR; ++f) {
    const bool is_a = f == 0 || f > TN;
    const int row = is_a ? arow[f == 0 ? 0 : f - TN] : brow[f - 1];
    fbase[f] = lds0 + (uint32_t)((is_a ? 0 : BM * 8) + row * 8) * 16;
  }
  bf16x8 af[2][TM], bfr[2][TN];
  // fragment f of k-step ks of the stage at byte offset `stage` into register buffer `to`
  auto read_frag = [&](uint32_t stage, int ks, int f, int to) __attribute__((always_inline)) {
    const u32x4 v = lds_read16_raw<0>(fbase[f] + (stage + (swz ^ (uint32_t)(ks * 32))));
    if (f == 0) af[to][0] = __builtin_bit_cast(bf16x8, v);
    else if (f <= TN) bfr[to][f - 1] = __builtin_bit_cast(bf16x8, v);
    else af[to][f - TN] = __builtin_bit_cast(bf16x8, v);
  };
  // The NL load instructions of a k-tile are spread, one behind an MFMA, over the NS MFMAs that follow the
  // barrier which frees their stage (the rest of the last k-step and the first k-step of the next k-tile):
  // issued together right behind the barrier they fill the vector-memory queue, and a wavefront that waits
  // there to issue a load cannot issue the MFMAs behind it either.
  constexpr int NL = IA + IB, NS = (NM - NB) + NM;
#pragma unroll
  for (int q = 0; q < NL; ++q) load_part(0, 0, q);
  tile_barrier();
  static_for<NL>([&](auto q_) __attribute__((always_inline)) {
    constexpr int q = decltype(q_)::value;
    if constexpr (q * NS / NL < NM - NB) load_part(1, 1, q);           // the part that k-step 3 would have issued
  });
#pragma unroll
  for (int f = 0; f < NR; ++f) read_frag(0, 0, f, 0);
  for (int kt = 0; kt < KT; ++kt) {
    const uint32_t cur = (uint32_t)(kt & 1) * STAGE * 16, nxt = (uint32_t)((kt + 1) & 1) * STAGE * 16;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      static_for<NM>([&](auto n_) __attribute__((always_inline)) {
        constexpr int n = decltype(n_)::value, i = n / TN, j = n % TN;
        constexpr int need = frag_need<TN>(n), prev = n == 0 ? -1 : frag_need_upto<TN>(n - 1);
        if (ks < 3) {
          // reads of step ks+1 issued so far in this step: those with k * NM / NR < n
          if constexpr (need > prev) lds_wait<NR - 1 - need + reads_before<NM, NR>(n, 0)>();
        } else {
          if constexpr (n < NB) { if constexpr (need > prev) lds_wait<NR - 1 - need>(); }
          if constexpr (n == NB) tile_barrier();           // every read of this k-tile has landed (lgkmcnt(0) precedes it)
        }
        __builtin_amdgcn_sched_barrier(0);               // the MFMA stays behind the wait for its fragments
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ks & 1][j], af[ks & 1][i], acc[i][j], 0, 0, 0);
        static_for<NR>([&](auto k_) __attribute__((always_inline)) {
          constexpr int k = decltype(k_)::value;
          if (ks < 3) { if constexpr (k * NM / NR == n) read_frag(cur, ks + 1, k, (ks + 1) & 1); }
          else { if constexpr (n >= NB && NB + k * (NM - NB) / NR == n) read_frag(nxt, 0, k, 0); }
        });
        static_for<NL>([&](auto q_) __attribute__((always_inline)) {
          constexpr int q = decltype(q_)::value, slot = q * NS / NL;       // MFMAs after the barrier
          if (ks == 3) { if constexpr (n >= NB && slot == n - NB) load_part(kt + 2, kt & 1, q); }
          else if (ks == 0) { if constexpr (slot == (NM - NB) + n) load_part(kt + 1, (kt + 1) & 1, q); }
        });
        __builtin_amdgcn_sched_barrier(0);               // keeps the MFMAs, reads, loads and waits in this order
      });
    }
  }
  lds_wait<0>();

  // Epilogue.  The MFMAs ran with the weight rows as the A operand, so a lane holds the output row
  // m = .. + lr and, per register quad q, the four consecutive columns n = .. + q*8 + lg*4 + (0..3).
  // The tile goes through LDS (free now) so that global memory sees whole rows: 16 bytes per lane,
  // consecutive lanes on consecutive addresses.  LDS rows are XOR-swizzled with the row index so that
  // neither the column-wise writes nor the row-wise reads conflict on banks.
  constexpr int NW = WGM * WGN;
  const bf16_t* bias = (const bf16_t*)e.bias;
  if constexpr (EPI == EPI_HEADS) {
    // Sections of `dim` columns, each stored per attention head (see HeadsArgs).  A plain section gets, per
    // output row, the sum of squares of (acc + bias) over this tile's columns, taken from the fp32
    // accumulators; its channel gains and 3D rotation are applied on the way out of the staging tile, where
    // a lane holds 8 consecutive channels of one row, so that the table and gain reads are contiguous
    // across lanes.  A transposed section is C^T already.
    constexpr int UPR = BN / 4, CPR = BN / 8, RPI = 64 / CPR;
    static_assert(BM * BN * 2 <= (BM + BN) * 256, "EPI_HEADS stages the whole tile at once");
    __shared__ float red[BM * WGN];                      // [row][wavefront column]: sums of squares
    const HeadSection sc = ha.sec[sec];
    const int64_t nsec = n0 - (int64_t)sec * ha.dim;     // first column of this tile inside its section
    const int hshift = ha.head_dim == 128 ? 7 : 6, hmask = ha.head_dim - 1;
    uint2* l8 = (uint2*)smem;
    __syncthreads();
    if (swapped) {
      // lane: channel row (weight row) nsec + wm*WM + i*32 + lr; register quad: 4 consecutive output rows m
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = wm * WM + i * 32 + lr;
        const float bvr = bias && n0 + row < N ? bf16_to_f32(bias[n0 + row]) : 0.f;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int nl = wn * WN + j * 32 + q * 8 + lg * 4;
            uint2 pk;
            pk.x = cvt_pk_bf16(acc[i][j][q * 4 + 0] + bvr, acc[i][j][q * 4 + 1] + bvr);
            pk.y = cvt_pk_bf16(acc[i][j][q * 4 + 2] + bvr, acc[i][j][q * 4 + 3] + bvr);
            l8[row * UPR + ((nl >> 2) ^ (row & 31))] = pk;
          }
      }
    } else {
      float ss[TM];
#pragma unroll
      for (int i = 0; i < TM; ++i) ss[i] = 0.f;
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
            const int row = wm * WM + i * 32 + lr;
            float v[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
              v[t] = acc[i][j][q * 4 + t] + bv[t];
              ss[i] += v[t] * v[t];
            }
            uint2 pk;
            pk.x = cvt_pk_bf16(v[0], v[1]);
            pk.y = cvt_pk_bf16(v[2], v[3]);
            l8[row * UPR + ((nl >> 2) ^ (row & 31))] = pk;
          }
        }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const float tot = ss[i] + __shfl_xor(ss[i], 32, 64);
        if (lg == 0) red[(wm * WM + i * 32 + lr) * WGN + wn] = tot;
      }
    }
    __syncthreads();
    if (!swapped && sc.ssq) {
      // one value per row and tile, tile-major so that rows are contiguous: ssq[tile in section][m]
      for (int row = tid; row < BM; row += NT) {
        float tot = 0.f;
#pragma unroll
        for (int w = 0; w < WGN; ++w) tot += red[row * WGN + w];
        if (m0 + row < M) sc.ssq[(nsec / BN) * ha.ssq_stride + m0 + row] = tot;
      }
    }
    // A lane always takes the same two logical chunks (8 consecutive columns each), BN / 2 columns apart, of
    // its rows, so its gains and channel-pair indices are fixed, and where BN / 2 is a multiple of the head
    // width both chunks rotate by the same table entries.  The loads of a group of rows (staging tile,
    // rotation table) are issued together.
    constexpr int HC = CPR / 2, RP2 = 64 / HC, IT = BM / NW / RP2, G = 4;
    static_assert(BM / NW % RP2 == 0, "rows per wavefront");
    const int c8 = (lane % HC) * 8;                      // first column of chunk 0; chunk 1 starts at c8 + BN / 2
    const bool rotate = !swapped && sc.rope, scale = !swapped && (sc.gain || sc.rope);
    const bool share = (BN / 2) % ha.head_dim == 0;      // both chunks use the same channel pairs
    const int half = ha.head_dim >> 1;
    float gg[2][8];
    int nn[2], p0[2];
    bool col_ok[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      nn[k] = (int)nsec + c8 + k * (BN / 2);             // first of the chunk's 8 channels inside the section
      p0[k] = (nn[k] & hmask) >> 1;
      col_ok[k] = n0 + c8 + k * (BN / 2) < N;
#pragma unroll
      for (int t = 0; t < 8; ++t) gg[k][t] = 1.f;
      if (!swapped && sc.gain && col_ok[k]) {
        const float4 g0 = *(const float4*)(sc.gain + nn[k]), g1 = *(const float4*)(sc.gain + nn[k] + 4);
        gg[k][0] = g0.x; gg[k][1] = g0.y; gg[k][2] = g0.z; gg[k][3] = g0.w;
        gg[k][4] = g1.x; gg[k][5] = g1.y; gg[k][6] = g1.z; gg[k][7] = g1.w;
      }
    }
#pragma unroll
    for (int it0 = 0; it0 < IT; it0 += G) {
      uint4 d[G][2];
      float4 cs[G][2][2];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        if (it0 + g < IT) {
          const int row = wave * (BM / NW) + (it0 + g) * RP2 + lane / HC;
#pragma unroll
          for (int k = 0; k < 2; ++k) {
            d[g][k] = smem[row * CPR + (((c8 >> 3) + k * HC) ^ ((row & 31) >> 1))];
            if (row & 1) d[g][k] = make_uint4(d[g][k].z, d[g][k].w, d[g][k].x, d[g][k].y);
          }
          if (rotate && m0 + row < M) {
            const float4* t = (const float4*)(ha.cs + (m0 + row) * half + p0[0]);
            cs[g][0][0] = t[0]; cs[g][0][1] = t[1];
            if (!share) {
              const float4* t1 = (const float4*)(ha.cs + (m0 + row) * half + p0[1]);
              cs[g][1][0] = t1[0]; cs[g][1][1] = t1[1];
            }
          }
        }
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        if (it0 + g < IT) {
          const int row = wave * (BM / NW) + (it0 + g) * RP2 + lane / HC;
#pragma unroll
          for (int k = 0; k < 2; ++k) {
            if (swapped) {
              const int64_t ch = nsec + row, m = m0 + c8 + k * (BN / 2);   // channel in the section, first of 8 output rows
              if (ch < ha.dim && n0 + row < N && m < M)
                __builtin_nontemporal_store(u32x4{d[g][k].x, d[g][k].y, d[g][k].z, d[g][k].w}, (u32x4*)((bf16_t*)sc.dst + ch * sc.ld + sc.row0 + m));
            } else if (m0 + row < M && col_ok[k]) {
              const int64_t m = m0 + row;
              uint4 dv = d[g][k];
              if (scale) {
                const uint32_t w[4] = {dv.x, dv.y, dv.z, dv.w};
                const float4 c0 = cs[g][share ? 0 : k][0], c1 = cs[g][share ? 0 : k][1];
                const float csv[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
                uint32_t o[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                  float a = bf16_to_f32((bf16_t)(w[u] & 0xffff)) * gg[k][2 * u], b = bf16_to_f32((bf16_t)(w[u] >> 16)) * gg[k][2 * u + 1];
                  if (rotate) {
                    const float a2 = a * csv[2 * u] - b * csv[2 * u + 1], b2 = a * csv[2 * u + 1] + b * csv[2 * u];
                    a = a2; b = b2;
                  }
                  o[u] = cvt_pk_bf16(a, b);
                }
                dv = make_uint4(o[0], o[1], o[2], o[3]);
              }
              // non-temporal like the other streamed outputs (same-box A/B, 14400 x 15360 x 5120: 1915 -> 1851 us)
              __builtin_nontemporal_store(u32x4{dv.x, dv.y, dv.z, dv.w}, (u32x4*)((bf16_t*)sc.dst + (int64_t)(nn[k] >> hshift) * sc.ld + (sc.row0 + m) * ha.head_dim + (nn[k] & hmask)));
            }
          }
        }
      }
    }
  } else if constexpr (EPI != EPI_RESID) {
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
        // streamed out once; non-temporal so that the output does not displace the operand panels the other
        // tiles still re-read from the caches (measured at the 14400 x 13824 x 5120 GELU shape: -3 %)
        if (m < M && n < N) __builtin_nontemporal_store(u32x4{d.x, d.y, d.z, d.w}, (u32x4*)((bf16_t*)e.out + m * e.ldo + n));
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
        // This wavefront's share of the group's residual rows is requested before the group is staged, so the
        // loads travel while the accumulators go through LDS (same-box A/B at 14400 x 5120 x 5120: 724 -> 679 us)
        constexpr int NIT = (GI * 32 + NW * RPI - 1) / (NW * RPI);
        float4 xpre[NIT];
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
          const int r = wave * RPI + it * NW * RPI;
          if (r < gi * 32) {
            const int row = r + lane / CPR, p = lane % CPR;
            const int64_t m = m0 + pass * WM + i0 * 32 + row, n = n0 + (p ^ (row & 15)) * 4;
            if (m < M && n < N) xpre[it] = *(const float4*)(e.resid + m * e.ldr + n);
          }
        }
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
        // gi * 32 rows, shared out over the wavefronts RPI rows per read; the residual values were requested
        // before the staging above, so they are on their way (or there) by now
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
          const int r = wave * RPI + it * NW * RPI;
          if (r < gi * 32) {
            const int row = r + lane / CPR, p = lane % CPR;
            const float4 v = l16[row * CPR + p];
            const int64_t m = m0 + pass * WM + i0 * 32 + row, n = n0 + (p ^ (row & 15)) * 4;
            if (m < M && n < N) {
              float4 xv = xpre[it];
              xv.x += v.x; xv.y += v.y; xv.z += v.z; xv.w += v.w;
              *(float4*)(e.resid + m * e.ldr + n) = xv;
              if (e.out) {
                uint2 pk;
                pk.x = cvt_pk_bf16(xv.x, xv.y);
                pk.y = cvt_pk_bf16(xv.z, xv.w);
                *(uint2*)((bf16_t*)e.out + m * e.ldo + n) = pk;
              }
            }
          }
        }
      }
    }
  }
}

template <int BM, int BN, int WGM, int WGN, int EPI>
static void launch_one(const bf16_t* A, int64_t lda, const bf16_t* Wt, int64_t ldw, int64_t M, int64_t N,
                       int64_t K, const EpiArgs& e, hipStream_t st) {
  constexpr int NT = WGM * WGN * 64;
  constexpr size_t lds = (size_t)(BM + BN) * 128 * 2;
  const int tm = (int)((M + BM - 1) / BM), tn = (int)((N + BN - 1) / BN);
  static std::atomic<uint64_t> done;
  allow_dynamic_lds((const void*)k_gemm_bf16<BM, BN, WGM, WGN, EPI>, (int)lds, done);
  HeadsArgs ha{};
  if (EPI == EPI_HEADS) { e.heads->ssq_np = e.heads->dim / BN; ha = *e.heads; }
  dim3 grid((unsigned)((tm * tn + 7) / 8 * 8));
  k_gemm_bf16<BM, BN, WGM, WGN, EPI><<<grid, NT, lds, st>>>(A, lda, Wt, ldw, M, N, K, tn, tm * tn, e, ha);
}
template <int BM, int BN, int WGM, int WGN>
static void launch_cfg(const bf16_t* A, int64_t lda, const bf16_t* Wt, int64_t ldw, int64_t M, int64_t N,
                       int64_t K, int epi, const EpiArgs& e, hipStream_t st) {
  if (epi == EPI_STORE) launch_one<BM, BN, WGM, WGN, EPI_STORE>(A, lda, Wt, ldw, M, N, K, e, st);
  else if (epi == EPI_GELU) launch_one<BM, BN, WGM, WGN, EPI_GELU>(A, lda, Wt, ldw, M, N, K, e, st);
  else launch_one<BM, BN, WGM, WGN, EPI_RESID>(A, lda, Wt, ldw, M, N, K, e, st);
}

// EPI_HEADS.  Sections must be whole tiles wide (dim % 256 == 0, or dim % 128 == 0 for problems small enough
// for 128x128 tiles) and a transposed section needs a square tile, 8 | M and 8 | row0.
bool gemm_bf16_heads_ok(int64_t M, int64_t N, const HeadsArgs& h) {
  const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256);
  const int bn = t256 < 64 ? 128 : 256;
  if (h.dim <= 0 || (h.head_dim != 64 && h.head_dim != 128) || h.dim % bn || h.dim % h.head_dim || N % h.dim || N / h.dim > 3) return false;
  for (int i = 0; i < (int)(N / h.dim); ++i) {
    if (h.sec[i].transposed && (M % 8 || h.sec[i].row0 % 8 || h.sec[i].ld % 8)) return false;
    if (h.sec[i].ssq && h.ssq_stride < M) return false;
  }
  return true;
}
static void launch_gemm_bf16_heads(const bf16_t* A, int64_t lda, const bf16_t* Wt, int64_t ldw, int64_t M, int64_t N,
                                   int64_t K, const EpiArgs& e, hipStream_t st) {
  const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256);
  if (t256 < 64) { launch_one<128, 128, 2, 2, EPI_HEADS>(A, lda, Wt, ldw, M, N, K, e, st); return; }
  bool any_t = false;
  for (int i = 0; i < (int)(N / e.heads->dim); ++i) any_t = any_t || e.heads->sec[i].transposed;
  // the 160-row tile cannot exchange its operands; it pays where it fills the one round better (see below)
  const int64_t t160 = ((M + 159) / 160) * ((N + 255) / 256);
  const bool fits160 = (M + 159) / 160 * 160 <= (M + 255) / 256 * 256;
  if (!any_t && fits160 && 0.80 * (double)((t160 + 255) / 256) < (double)((t256 + 255) / 256))
    launch_one<160, 256, 1, 8, EPI_HEADS>(A, lda, Wt, ldw, M, N, K, e, st);
  else
    launch_one<256, 256, 2, 4, EPI_HEADS>(A, lda, Wt, ldw, M, N, K, e, st);
}

bool launch_gemm_bf16(const bf16_t* A, int64_t lda, const bf16_t* Wt, int64_t ldw, int64_t M, int64_t N,
                      int64_t K, int epi, const EpiArgs& e, hipStream_t st) {
  if (M <= 0 || N <= 0) return true;
  if (K < 64 || K % 64) return false;          // whole k-tiles of 64 (the callers validate their widths)
  if (epi == EPI_HEADS) {
    if (!e.heads || !gemm_bf16_heads_ok(M, N, *e.heads)) return false;
    launch_gemm_bf16_heads(A, lda, Wt, ldw, M, N, K, e, st);
    return true;
  }
  // One block per CU at a time, so a launch costs ceil(blocks / 256) rounds of one block's duration.
  // 256x256 tiles are the default.  Other shapes are taken when rounds x relative duration comes out lower:
  // 192x256 (0.88 of a 256x256 tile), 160x256 (0.80; 1 x 8 wavefronts, more LDS reads per MFMA, but e.g. 39 x 6
  // tiles fill one round where 33 x 6 leave 58 CUs idle) and 320x256 (1.25, fewer operand bytes per flop).
  // The 160-, 192- and 320-row tiles read rows beyond M up to their own multiple, so they are used only where
  // that stays inside the 256-row padding the caller guarantees.  Tiny problems take 128x128 tiles.
  const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256);
  const int64_t t192 = ((M + 191) / 192) * ((N + 255) / 256);
  const int64_t t160 = ((M + 159) / 160) * ((N + 255) / 256);
  const int64_t t320 = ((M + 319) / 320) * ((N + 255) / 256);
  if (t256 < 64) { launch_cfg<128, 128, 2, 2>(A, lda, Wt, ldw, M, N, K, epi, e, st); return true; }
  const int64_t mpad = (M + 255) / 256 * 256;
  const double cost256 = (double)((t256 + 255) / 256);
  const double cost192 = (M + 191) / 192 * 192 <= mpad ? 0.88 * (double)((t192 + 255) / 256) : 1e30;
  const double cost160 = (M + 159) / 160 * 160 <= mpad ? 0.80 * (double)((t160 + 255) / 256) : 1e30;
  const double cost320 = (M + 319) / 320 * 320 <= mpad ? 1.25 * (double)((t320 + 255) / 256) : 1e30;
  const double best = fmin(fmin(cost256, cost192), fmin(cost160, cost320));
  // on a tie the taller tile wins: fewer operand bytes per flop
  if (best == cost320) { launch_cfg<320, 256, 2, 4>(A, lda, Wt, ldw, M, N, K, epi, e, st); return true; }
  if (best == cost256) { launch_cfg<256, 256, 2, 4>(A, lda, Wt, ldw, M, N, K, epi, e, st); return true; }
  if (best == cost160) { launch_cfg<160, 256, 1, 8>(A, lda, Wt, ldw, M, N, K, epi, e, st); return true; }
  launch_cfg<192, 256, 2, 4>(A, lda, Wt, ldw, M, N, K, epi, e, st);
  return true;
}
