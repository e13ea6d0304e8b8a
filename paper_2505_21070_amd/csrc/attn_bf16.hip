// Flash attention on the gfx950 matrix cores for the DP_BF16 path: the block's queries attend over one
// contiguous key range [cached prefix ; current block] streamed from HBM through LDS tiles, with an
// online softmax in fp32.  Used for self-attention (cache + block) and cross-attention (text keys).
//
// Scores are computed transposed, S^T = K * Q^T (keys are MFMA rows, queries MFMA columns): a lane
// then owns one query column, so the softmax maximum and sum are reductions over the lane's own
// registers plus one exchange with lane ^ 32, and the fp32 S^T accumulators, once exponentiated and
// rounded to bf16, ARE the B operand of the second product O^T = V^T * P^T.  The rows of a K tile are
// stored in a permuted order so that the eight accumulators a lane packs into one operand belong to
// eight consecutive keys, which makes the matching V^T operand one plain 16-byte LDS read.
//
// Q arrives pre-multiplied by log2(e)/sqrt(head_dim), so scores are base-2 logits.  The softmax reference
// m of a query is folded into the accumulator that the score MFMAs start from (-m instead of 0), so the
// matrix cores hand back s - m and the vector unit only has to exponentiate.  Fast pass: m is fixed once,
// to the query's maximum over the first 32 keys of its key group, and never raised, so O^T needs no
// rescaling and the loop body is straight-line code.  This is exact as long as nothing overflows: P (bf16)
// and the fp32 sums have 8 exponent bits, so scores may exceed m by ~2^100 before anything is lost.  A
// block whose row sums end up beyond 2^100 (or non-finite) is recomputed by the safe pass, the classical
// online softmax that raises m whenever a tile exceeds it and rescales O^T.
//
// Work split: a block of 8 wavefronts owns QG * 32 queries of one head.  Two shapes are built.
// QG = 4, KG = 2 (few queries or very few keys): wavefront w handles query tile w & 3 against key group
// w >> 2 (first / second half of the key tiles); the two groups stream their own K / V^T tiles and are
// merged through LDS at the end, which halves the length of a block.  QG = 8, KG = 1 (everything else,
// self- and cross-attention at full size): all 8 wavefronts share every K / V^T tile, so a tile brought
// into LDS serves 256 queries and the LDS fill traffic per query halves.  Tiles hold 64 keys, are double-buffered and are loaded
// HBM -> LDS directly.  The two wavefronts of a SIMD are served oldest first rather than interleaved, so the
// fast pass pins its issue order so that one wavefront alone keeps the matrix pipe busy: exponentials
// between MFMAs, operand fragments read from LDS several MFMAs ahead with exact waits (see pass_fast).
//
// Grid: one block fits per compute unit, so a grid runs in rounds of 256 blocks.  The work ids that
// would make up a last, partly filled round are instead cut into several key ranges each, one block per
// range, which write unnormalised partial results (m, l, O) to a scratch buffer; k_attn_merge joins them.
#include <type_traits>

#include "kernels.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void glb_void_t;

__device__ __forceinline__ uint32_t cvt_pk_bf16(float a, float b) {
  f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
// acc + lo + hi of a packed bf16 pair
__device__ __forceinline__ float add_pk_bf16(uint32_t pk, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk), __builtin_bit_cast(bf16x2, 0x3f803f80u), acc, false);
}
// LDS has 64 four-byte banks: 16 lanes x 16 bytes are served per cycle.  XOR-swizzling the 16-byte chunk
// index with the row spreads a column of chunks over all banks: rows of 256 bytes use row & 15, rows of
// 128 bytes (two rows per bank sweep) use (row >> 1) & 7.
template <int CR> __device__ __forceinline__ int kswz(int row) { return CR == 16 ? (row & 15) : ((row >> 1) & 7); }
// tile row -> key held in that row: bits 2 and 3 of the row index are exchanged
__device__ __forceinline__ int swap23(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

template <int OFF> __device__ __forceinline__ bf16x8 lds_read16(uint32_t addr) {
  return __builtin_bit_cast(bf16x8, lds_read16_raw<OFF>(addr));
}

template <int HD, int QG, int KG>
__global__ __launch_bounds__(512) void k_attn_bf16(const bf16_t* __restrict__ q, int64_t q_head_stride,
                                                  const bf16_t* __restrict__ k, int64_t k_head_stride,
                                                  int64_t k_row0, const bf16_t* __restrict__ vt,
                                                  int64_t vt_row_stride, int64_t S, int64_t L,
                                                  bf16_t* __restrict__ out, int64_t ldo, int qblocks,
                                                  int n_full, int n_tail, int parts,
                                                  float* __restrict__ partial, AttnQNorm qn) {
  constexpr int CR = HD / 8;                 // 16-byte chunks per K row
  constexpr int KS = HD / 16;                // MFMA k-steps over the head dim
  constexpr int DT = HD / 32;                // 32-row tiles of O^T
  constexpr int KCH = 64 * CR;               // chunks in a K tile
  constexpr int VCH = HD * 8;                // chunks in a V^T tile
  constexpr int NBUF = 2;                    // tile buffers per key group (a third one was measured: no gain)
  constexpr int GCH = NBUF * (KCH + VCH);    // chunks per key group: NBUF K tiles, NBUF V^T tiles
  constexpr int CK = KCH / (QG * 64), CV = VCH / (QG * 64);   // load instructions per wavefront and tile
  constexpr int QB = QG * 32;                // queries per block
  static_assert(QG * KG == 8, "8 wavefronts");
  extern __shared__ uint4 smem[];            // KG * GCH chunks

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qt = wave % QG, kg = wave / QG;
  const int lr = lane & 31, lg = lane >> 5;
  // Blocks are dealt round-robin over the 8 XCDs, each with its own L2: give every XCD a contiguous run
  // of (head, query block) work ids so that the blocks streaming one head's K/V share an L2.  The first
  // n_full blocks (a multiple of 8) each own a whole work id; the n_tail work ids after them are cut into
  // `parts` key ranges each, one block per range, again padded to a multiple of 8 blocks that have nothing
  // to do.
  const int NKT = (int)((L + 63) / 64);
  int wid, t0 = 0, t1 = NKT, slot = -1;
  if ((int)blockIdx.x < n_full) {
    wid = (int)(blockIdx.x & 7) * (n_full >> 3) + (int)(blockIdx.x >> 3);
  } else {
    const int local = (int)blockIdx.x - n_full, tail_grid = (int)gridDim.x - n_full;
    const int pid = (local & 7) * (tail_grid >> 3) + (local >> 3);
    if (pid >= n_tail * parts) return;
    wid = n_full + pid / parts;
    if (parts > 1) {
      const int part = pid % parts;
      t0 = (int)((int64_t)part * NKT / parts);
      t1 = (int)((int64_t)(part + 1) * NKT / parts);
      slot = pid;
    }
  }
  const int head = wid / qblocks;
  const int64_t q0 = (int64_t)(wid % qblocks) * QB + qt * 32;
  uint4* const kbuf = smem + kg * GCH;
  uint4* const vbuf = kbuf + NBUF * KCH;

  // this wavefront's share of the key tiles
  const int n0 = KG == 2 ? (t1 - t0 + 1) / 2 : t1 - t0;   // tiles of group 0; also the trip count for everyone
  const int first = t0 + (kg ? n0 : 0), cnt = kg ? t1 - t0 - n0 : n0;

  // Q fragments stay in registers: B operand, column = query, 8 head-dim values per lane
  bf16x8 qf[KS];
  {
    const bf16_t* qh = q + (int64_t)head * q_head_stride + (q0 + lr) * HD + lg * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, *(const uint4*)(qh + ks * 16));
  }
  if (qn.ssq) {
    // deferred RMSNorm of the queries: the row's sum of squares arrives as qn.np partial sums; the two lanes
    // that share a query row add up the even and the odd ones
    const int64_t row = q0 + lr < S ? q0 + lr : S - 1;
    const float* pr = qn.ssq + row;
    float sum = 0.f;
#pragma unroll 4
    for (int i = lg; i < qn.np; i += 2) sum += pr[i * qn.stride];
    sum += __shfl_xor(sum, 32, 64);
    const float r = rsqrtf(sum * qn.inv_dim + qn.eps) * qn.scale;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[ks][e] = (__bf16)((float)qf[ks][e] * r);
  }
  const bf16_t* kh = k + (int64_t)head * k_head_stride + (k_row0 + (int64_t)first * 64) * HD;
  const bf16_t* vh = vt + (int64_t)head * HD * vt_row_stride + k_row0 + (int64_t)first * 64;

  // HBM -> LDS directly (no staging registers).  One wavefront instruction fills 64 consecutive
  // 16-byte LDS slots, slot = base + lane; each lane fetches the chunk that belongs in its slot:
  // K slot p holds chunk (p % CR) ^ kswz(row) of key swap23(row), row = p / CR;
  // V^T slot p holds chunk (p % 8) ^ ((row >> 1) & 7) of channel row = p / 8.
  int koff[CK], voff[CV];
#pragma unroll
  for (int i = 0; i < CK; ++i) {
    const int p = qt * (KCH / QG) + i * 64 + lane, row = p / CR, ch = (p % CR) ^ kswz<CR>(row);
    koff[i] = swap23(row) * HD + ch * 8;
  }
#pragma unroll
  for (int i = 0; i < CV; ++i) {
    const int p = qt * (VCH / QG) + i * 64 + lane, row = p >> 3, ch = (p & 7) ^ ((row >> 1) & 7);
    voff[i] = row * (int)vt_row_stride + ch * 8;
  }
  // load instruction i of this wavefront's share of a tile: the K part first (i < CK), then the V^T part
  auto load_part = [&](int tile, int bufi, int i) __attribute__((always_inline)) {
    if (i < CK)
      __builtin_amdgcn_global_load_lds((glb_void_t*)(kh + (int64_t)tile * 64 * HD + koff[i]),
                                       (lds_void_t*)(kbuf + bufi * KCH + qt * (KCH / QG) + i * 64), 16, 0, 0);
    else
      __builtin_amdgcn_global_load_lds((glb_void_t*)(vh + (int64_t)tile * 64 + voff[i - CK]),
                                       (lds_void_t*)(vbuf + bufi * VCH + qt * (VCH / QG) + (i - CK) * 64), 16, 0, 0);
  };
  auto load_tile = [&](int tile, int bufi) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < CK + CV; ++i) load_part(tile, bufi, i);
  };

  f32x16 oacc[DT], negm;
  float mrun, lsum;

  // One pass over this wavefront's key tiles.  SAFE = false: fixed reference (see the file header).
  // SAFE = true: classical online softmax, reference raised per 32-key half tile, O^T rescaled.
  auto pass = [&](auto safe_tag) __attribute__((always_inline)) {
    constexpr bool SAFE = decltype(safe_tag)::value;
#pragma unroll
    for (int a = 0; a < DT; ++a)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[a][r] = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) negm[r] = 0.f;
    mrun = 0.f; lsum = 0.f;
    bool fresh = true;                                  // SAFE: no key seen yet, mrun is a placeholder

    if (cnt > 0) load_tile(0, 0);
    tile_barrier();
    if (!SAFE && cnt > 0) {
      // reference = maximum over the first 32 keys (all valid: a group's first tile starts below L)
      f32x16 s0;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int row = lr, ch = ks * 2 + lg;
        const bf16x8 kf = __builtin_bit_cast(bf16x8, kbuf[row * CR + (ch ^ kswz<CR>(row))]);
        s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], ks == 0 ? negm : s0, 0, 0, 0);
      }
      const int kv0 = (int)(L - (int64_t)first * 64);
      float mx = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (swap23((r >> 2) * 8 + lg * 4 + (r & 3)) < kv0) mx = fmaxf(mx, s0[r]);
      mrun = fmaxf(mx, __shfl_xor(mx, 32, 64));
#pragma unroll
      for (int r = 0; r < 16; ++r) negm[r] = -mrun;
    }

    for (int kt = 0; kt < n0; ++kt) {
      if (kt < cnt) {
        // next tile into the other buffer (read last before the previous barrier); the tile past the
        // end is the last one again and never used
        load_tile(kt + NBUF - 1 < cnt ? kt + NBUF - 1 : cnt - 1, (kt + NBUF - 1) % NBUF);
        const uint4* kb = kbuf + (kt % NBUF) * KCH;
        const uint4* vb = vbuf + (kt % NBUF) * VCH;
        const int kvalid = (int)(L - (int64_t)(first + kt) * 64);     // < 64 only in the ragged last tile
#pragma unroll
        for (int a = 0; a < 2; ++a) {                                  // two 32-key halves of the tile
          // S^T - m : 32 keys x 32 queries, accumulation started from -m
          f32x16 sacc;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            const int row = a * 32 + lr, ch = ks * 2 + lg;
            const bf16x8 kf = __builtin_bit_cast(bf16x8, kb[row * CR + (ch ^ kswz<CR>(row))]);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], ks == 0 ? negm : sacc, 0, 0, 0);
          }
          // register r, lane group lg, is tile row a*32 + (r/4)*8 + lg*4 + (r%4), which holds key
          // swap23(row); keys at or beyond L get -inf
          if (kvalid < 64) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
              if (swap23(a * 32 + (r >> 2) * 8 + lg * 4 + (r & 3)) >= kvalid) sacc[r] = -INFINITY;
          }
          if constexpr (SAFE) {
            float mx = sacc[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sacc[r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));                    // maximum of this half relative to m
            const float up = fresh ? mx : fmaxf(mx, 0.f);
            const float alpha = fresh ? 0.f : __builtin_amdgcn_exp2f(-up);
            mrun += up;
            lsum *= alpha;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
              for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
#pragma unroll
            for (int r = 0; r < 16; ++r) { sacc[r] -= up; negm[r] = -mrun; }
            fresh = false;
          }
          // P = 2^(s - m), packed to bf16 as the B operand of O^T += V^T P^T; row sums from the rounded values
          uint4 pf[2];
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            uint32_t w[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              w[j] = cvt_pk_bf16(__builtin_amdgcn_exp2f(sacc[u * 8 + 2 * j]), __builtin_amdgcn_exp2f(sacc[u * 8 + 2 * j + 1]));
              lsum = add_pk_bf16(w[j], lsum);
            }
            pf[u] = make_uint4(w[0], w[1], w[2], w[3]);
          }
          // O^T += V^T * P^T : k-step u covers keys [a*32 + 16u, +16), lane group lg the lower/upper 8
#pragma unroll
          for (int u = 0; u < 2; ++u) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
              const int row = dt * 32 + lr, ch = (a * 2 + u) * 2 + lg;
              const bf16x8 vf = __builtin_bit_cast(bf16x8, vb[row * 8 + (ch ^ ((row >> 1) & 7))]);
              oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, __builtin_bit_cast(bf16x8, pf[u]), oacc[dt], 0, 0, 0);
            }
          }
        }
      }
      tile_barrier();       // the next tile has landed and every wavefront is done with this one
    }
    return fresh;
  };


  // Fast pass (fixed reference).  Per tile a wavefront issues NMF MFMAs in the order S^T of the first 32-key
  // half, S^T of the second half, O^T += V^T P^T of the first half, then of the second; the exponentials of
  // the first half are issued between the MFMAs of the second half's S^T and those of the second half
  // between the first half's V^T P^T MFMAs, so the vector unit works while the matrix pipe runs.  Every MFMA
  // takes one operand fragment from LDS; fragment i + PD is read right behind MFMA i, through inline
  // assembly with explicit waits (LDS returns reads in order), so an MFMA never waits for a read issued
  // just before it.  The tile's barrier sits PD MFMAs before the tile's end, once all its fragments are in
  // registers: behind it the loads of the tile after next and the first PD fragment reads of the next tile
  // go out between the remaining MFMAs.
  constexpr int NMF = 2 * (KS + 2 * DT), PD = 4, PPM = 8 / KS;      // MFMAs per tile, read-ahead, exp pairs per MFMA
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_void_t*)smem;
  // This lane's row of a K tile (row lr of a 32-key half) and of a V^T tile (row lr of a 32-channel group) in
  // buffer 0, as LDS byte addresses; chunk c of the row sits at byte (c * 16) ^ swizzle, and c = ks*2 + lg or
  // (a*2+u)*2 + lg has lg as its lowest bit, so the lane-dependent part of the XOR is one constant per tile kind.
  const uint32_t krow = lds0 + (uint32_t)(kg * GCH + lr * CR) * 16, kx = (uint32_t)(lg ^ kswz<CR>(lr)) * 16;
  const uint32_t vrow = lds0 + (uint32_t)(kg * GCH + NBUF * KCH + lr * 8) * 16, vx = (uint32_t)(lg ^ ((lr >> 1) & 7)) * 16;
  // operand fragment of MFMA i of a tile whose K / V^T buffers start kbo / vbo bytes behind buffer 0
  auto frag_read = [&](auto i_, uint32_t kbo, uint32_t vbo) __attribute__((always_inline)) {
    constexpr int i = decltype(i_)::value;
    if constexpr (i < 2 * KS) {
      return lds_read16<(i / KS) * 32 * CR * 16>((krow + kbo) + (kx ^ (uint32_t)((i % KS) * 32)));
    } else {
      constexpr int j = i - 2 * KS, a = j / (2 * DT), u = (j % (2 * DT)) / DT, dt = j % DT;
      return lds_read16<dt * 32 * 8 * 16>((vrow + vbo) + (vx ^ (uint32_t)((a * 2 + u) * 32)));
    }
  };
  auto pass_fast = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int a = 0; a < DT; ++a)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[a][r] = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) negm[r] = 0.f;
    mrun = 0.f; lsum = 0.f;
    // Step j of this pass works on tile cnt - 1 - j of the range (the sums do not care about the order), in
    // buffer j % NBUF: the last tile of the range, the only one that can be ragged, comes first and is done
    // here in plain order with its keys at or beyond L masked; the pinned loop below then sees whole tiles only.
    if (cnt > 0) load_tile(cnt - 1, 0);
    if (cnt > 1) load_tile(cnt - 2, 1);
    tile_barrier();
    if (cnt > 0) {
      const int kvalid = (int)(L - (int64_t)(first + cnt - 1) * 64);   // >= 1; < 64 only in a ragged tile
      // reference = maximum over the tile's first 32 keys (the valid ones of them).  Register r of lane group
      // lg is tile row a*32 + (r/4)*8 + lg*4 + r%4, which holds key swap23(row).
      f32x16 sv;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int row = lr, ch = ks * 2 + lg;
        const bf16x8 kf = __builtin_bit_cast(bf16x8, kbuf[row * CR + (ch ^ kswz<CR>(row))]);
        sv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], ks == 0 ? negm : sv, 0, 0, 0);
      }
      float mx = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (swap23((r >> 2) * 8 + lg * 4 + (r & 3)) < kvalid) mx = fmaxf(mx, sv[r]);
      mrun = fmaxf(mx, __shfl_xor(mx, 32, 64));
#pragma unroll
      for (int r = 0; r < 16; ++r) negm[r] = -mrun;
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        if (a == 0) {
#pragma unroll
          for (int r = 0; r < 16; ++r) sv[r] -= mrun;
        } else {
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            const int row = 32 + lr, ch = ks * 2 + lg;
            const bf16x8 kf = __builtin_bit_cast(bf16x8, kbuf[row * CR + (ch ^ kswz<CR>(row))]);
            sv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], ks == 0 ? negm : sv, 0, 0, 0);
          }
        }
        if (kvalid < 64) {
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (swap23(a * 32 + (r >> 2) * 8 + lg * 4 + (r & 3)) >= kvalid) sv[r] = -INFINITY;
        }
        uint4 pf[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          uint32_t w[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            w[j] = cvt_pk_bf16(__builtin_amdgcn_exp2f(sv[u * 8 + 2 * j]), __builtin_amdgcn_exp2f(sv[u * 8 + 2 * j + 1]));
            lsum = add_pk_bf16(w[j], lsum);
          }
          pf[u] = make_uint4(w[0], w[1], w[2], w[3]);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) {
            const int row = dt * 32 + lr, ch = (a * 2 + u) * 2 + lg;
            const bf16x8 vf = __builtin_bit_cast(bf16x8, vbuf[row * 8 + (ch ^ ((row >> 1) & 7))]);
            oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, __builtin_bit_cast(bf16x8, pf[u]), oacc[dt], 0, 0, 0);
          }
      }
    }
    tile_barrier();                 // every wavefront is done with buffer 0
    if (cnt > 2) load_tile(cnt - 3, 0);
    bf16x8 fr[PD];
    f32x16 sacc[2];
    uint32_t pw[2][8];              // P of the two halves: packed bf16 pairs, four per MFMA operand
    static_for<PD>([&](auto i_) __attribute__((always_inline)) {
      fr[decltype(i_)::value] = frag_read(i_, (uint32_t)(1 % NBUF) * KCH * 16, (uint32_t)(1 % NBUF) * VCH * 16);
    });
    // exponentials of scores 2p, 2p+1 of half a, packed; row sums from the rounded values
    auto e_piece = [&](int a, int pidx) __attribute__((always_inline)) {
      pw[a][pidx] = cvt_pk_bf16(__builtin_amdgcn_exp2f(sacc[a][2 * pidx]), __builtin_amdgcn_exp2f(sacc[a][2 * pidx + 1]));
      lsum = add_pk_bf16(pw[a][pidx], lsum);
    };
    for (int j = 1; j < n0; ++j) {
      if (j < cnt) {
        const uint32_t kbo = (uint32_t)(j % NBUF) * KCH * 16, vbo = (uint32_t)(j % NBUF) * VCH * 16;
        const uint32_t kbn = (uint32_t)((j + 1) % NBUF) * KCH * 16, vbn = (uint32_t)((j + 1) % NBUF) * VCH * 16;
        static_for<NMF>([&](auto i_) __attribute__((always_inline)) {
          constexpr int i = decltype(i_)::value;
          if constexpr (i < NMF - PD) lds_wait<PD - 1>();               // fragment i has landed
          __builtin_amdgcn_sched_barrier(0);                            // the MFMA stays behind the wait
          if constexpr (i < KS) {
            sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % PD], qf[i], i == 0 ? negm : sacc[0], 0, 0, 0);
          } else if constexpr (i < 2 * KS) {
            sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % PD], qf[i - KS], i == KS ? negm : sacc[1], 0, 0, 0);
#pragma unroll
            for (int e = 0; e < PPM; ++e) e_piece(0, (i - KS) * PPM + e);
          } else {
            constexpr int m = i - 2 * KS, a = m / (2 * DT), u = (m % (2 * DT)) / DT, dt = m % DT;
            const uint4 pf = make_uint4(pw[a][u * 4], pw[a][u * 4 + 1], pw[a][u * 4 + 2], pw[a][u * 4 + 3]);
            oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % PD], __builtin_bit_cast(bf16x8, pf), oacc[dt], 0, 0, 0);
            if constexpr (a == 0) {
#pragma unroll
              for (int e = 0; e < PPM; ++e) e_piece(1, m * PPM + e);
            }
          }
          // the two dependent S^T chains go first in the SIMD's issue arbitration (measured: 2 % over no hint)
          if constexpr (i == 0) __builtin_amdgcn_s_setprio(1);
          if constexpr (i == 2 * KS - 1) __builtin_amdgcn_s_setprio(0);
          __builtin_amdgcn_sched_barrier(0);      // the read that reuses the MFMA's operand register stays behind it
          if constexpr (i + PD < NMF) fr[i % PD] = frag_read(std::integral_constant<int, i + PD>{}, kbo, vbo);
          if constexpr (i == NMF - PD - 1) {
            lds_wait<0>();          // every fragment of this tile is in registers
            tile_barrier();         // the next tile has landed and every wavefront is done reading this one
          }
          if constexpr (i >= NMF - PD) {
            if (j + 2 < cnt) {
#pragma unroll
              for (int q = 0; q < CK + CV; ++q)
                if (q * PD / (CK + CV) == i - (NMF - PD)) load_part(cnt - 3 - j, j % NBUF, q);
            }
            fr[i % PD] = frag_read(std::integral_constant<int, i + PD - NMF>{}, kbn, vbn);
          }
          __builtin_amdgcn_sched_barrier(0);                            // keeps this order
        });
      } else {
        tile_barrier();
      }
    }
    lds_wait<0>();
  };

  pass_fast();
  const bool empty = cnt == 0;                          // this key group has no tile (a single-tile key range)
  float ltot = lsum + __shfl_xor(lsum, 32, 64);
  if (__syncthreads_or(!empty && !(ltot <= 0x1p100f))) {  // overflow somewhere in the block: redo it safely
    pass(std::true_type{});
    ltot = lsum + __shfl_xor(lsum, 32, 64);
  }

  // merge the two key groups through LDS (tile buffers are free now): group 1 publishes m, l, O^T
  float* xch = (float*)smem;                           // [qt][DT*16 + 2][64 lanes]
  float* mine = xch + (size_t)qt * (DT * 16 + 2) * 64 + lane;
  if constexpr (KG == 2) {
    if (kg == 1) {
      mine[0] = empty ? -INFINITY : mrun;
      mine[64] = ltot;
#pragma unroll
      for (int a = 0; a < DT; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) mine[(2 + a * 16 + r) * 64] = oacc[a][r];
    }
    __syncthreads();
  }
  if (kg == 0) {
    float m = mrun, a0 = 1.f, a1 = 0.f, lall = ltot;
    if constexpr (KG == 2) {
      const float m1 = mine[0], l1 = mine[64];
      const float m0 = empty ? -INFINITY : mrun;
      m = fmaxf(m0, m1);
      a0 = __builtin_amdgcn_exp2f(m0 - m); a1 = __builtin_amdgcn_exp2f(m1 - m);   // 2^-inf = 0
      lall = ltot * a0 + l1 * a1;
    }
    // this lane's O^T value (register r of channel tile a) over both key groups, scaled by w0 / w1
    auto both = [&](int a, int r, float w0, float w1) __attribute__((always_inline)) {
      float v = oacc[a][r] * w0;
      if constexpr (KG == 2) v += mine[(2 + a * 16 + r) * 64] * w1;
      return v;
    };
    const int64_t qi = q0 + lr;
    if (slot >= 0) {
      // one key range of a split work id: publish m, l and the unnormalised O^T for the merge kernel.
      // Slot layout (floats): m[QB], l[QB], then O as [HD/4][QB queries][4 channels].
      float* ps = partial + (size_t)slot * (2 * QB + QB * HD);
      const int ql = qt * 32 + lr;
      if (lg == 0) { ps[ql] = m; ps[QB + ql] = lall; }
#pragma unroll
      for (int a = 0; a < DT; ++a)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          float4 v;
          v.x = both(a, g4 * 4 + 0, a0, a1);
          v.y = both(a, g4 * 4 + 1, a0, a1);
          v.z = both(a, g4 * 4 + 2, a0, a1);
          v.w = both(a, g4 * 4 + 3, a0, a1);
          *(float4*)(ps + 2 * QB + ((size_t)(a * 8 + g4 * 2 + lg) * QB + ql) * 4) = v;
        }
    } else {
      // O[q][head*HD + c] = O^T[c][q]: a lane holds 4 consecutive channels per register quad.  The 32 x HD
      // tile of this wavefront goes through LDS (the tile buffers are free; a wavefront only touches its own
      // rows, and LDS serves a wavefront's accesses in order) so that global memory sees whole rows, 16
      // bytes per lane.  8-byte units are XOR-swizzled with the row so that the column-wise writes spread
      // over the banks.
      const float inv = 1.f / lall;
      const float w0 = a0 * inv, w1 = a1 * inv;
      constexpr int UPR = HD / 4, CPR = HD / 8, RPI = 64 / CPR;      // units, 16-byte chunks per row; rows per read
      constexpr int STG0 = KG == 2 ? QG * (DT * 16 + 2) * 64 * 4 / 16 : 0;    // behind the exchange area
      uint2* stg = (uint2*)(smem + STG0) + qt * 32 * UPR;
#pragma unroll
      for (int a = 0; a < DT; ++a)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          uint2 pk;
          pk.x = cvt_pk_bf16(both(a, g4 * 4 + 0, w0, w1), both(a, g4 * 4 + 1, w0, w1));
          pk.y = cvt_pk_bf16(both(a, g4 * 4 + 2, w0, w1), both(a, g4 * 4 + 3, w0, w1));
          stg[lr * UPR + ((a * 8 + g4 * 2 + lg) ^ (lr & (UPR - 1)))] = pk;
        }
      const uint4* stg16 = (const uint4*)stg;
#pragma unroll
      for (int it = 0; it < 32 / RPI; ++it) {
        const int row = it * RPI + lane / CPR, p = lane % CPR;
        uint4 dv = stg16[row * CPR + p];
        // units 2p and 2p+1 of the swizzled row are the halves of chunk p ^ (swizzle >> 1), exchanged for odd rows
        if (row & 1) dv = make_uint4(dv.z, dv.w, dv.x, dv.y);
        const int c = p ^ ((row & (UPR - 1)) >> 1);
        if (q0 + row < S) *(uint4*)(out + (q0 + row) * ldo + (int64_t)head * HD + c * 8) = dv;
      }
    }
  }
}

// Combines the key ranges of the split work ids: O = sum_i 2^(m_i - m) O_i / sum_i 2^(m_i - m) l_i with
// m = max_i m_i.  One thread per (query, 4 channels).  A block of 256 threads covers all channels of
// 256 / (HD/4) consecutive queries (query index fastest), so that partials are read in whole 128-byte
// lines and every output row is written from one block.
template <int HD, int QB>
__global__ __launch_bounds__(256) void k_attn_merge(const float* __restrict__ partial, int n_full, int n_tail,
                                                    int parts, int qblocks, int64_t S,
                                                    bf16_t* __restrict__ out, int64_t ldo) {
  constexpr int C4 = HD / 4, QPB = 256 / C4, SLOT = 2 * QB + QB * HD;
  const int tid = (int)threadIdx.x;
  const int gq = (int)blockIdx.x * QPB + tid % QPB;      // query index over all split work ids
  const int j = gq / QB, ql = gq % QB, c4 = tid / QPB;
  if (j >= n_tail) return;
  const int wid = n_full + j, head = wid / qblocks;
  const int64_t qi = (int64_t)(wid % qblocks) * QB + ql;
  if (qi >= S) return;
  const float* ps = partial + (size_t)j * parts * SLOT;
  float m = -INFINITY;
  for (int i = 0; i < parts; ++i) m = fmaxf(m, ps[(size_t)i * SLOT + ql]);
  float l = 0.f, o0 = 0.f, o1 = 0.f, o2 = 0.f, o3 = 0.f;
  for (int i = 0; i < parts; ++i) {
    const float* pi = ps + (size_t)i * SLOT;
    const float w = __builtin_amdgcn_exp2f(pi[ql] - m);
    const float4 v = *(const float4*)(pi + 2 * QB + ((size_t)c4 * QB + ql) * 4);
    l += w * pi[QB + ql];
    o0 += w * v.x; o1 += w * v.y; o2 += w * v.z; o3 += w * v.w;
  }
  const float inv = 1.f / l;
  uint2 pk;
  pk.x = cvt_pk_bf16(o0 * inv, o1 * inv);
  pk.y = cvt_pk_bf16(o2 * inv, o3 * inv);
  *(uint2*)(out + qi * ldo + (int64_t)head * HD + c4 * 4) = pk;
}

// partial results of at most 256 blocks of at most 256 queries
size_t attn_bf16_scratch_bytes(int d) { return (size_t)256 * (512 + 256 * (size_t)d) * sizeof(float); }

template <int HD, int QG, int KG>
static void launch_attn_cfg(const bf16_t* q, int64_t q_head_stride, const bf16_t* k, int64_t k_head_stride,
                            int64_t k_row0, const bf16_t* vt, int64_t vt_row_stride, int64_t S, int64_t L,
                            int h, bf16_t* out, int64_t ldo, float* scratch, const AttnQNorm& qn, hipStream_t st) {
  constexpr int QB = QG * 32;
  constexpr int lds = KG * 2 * (64 * (HD / 8) + HD * 8) * 16;
  const int qblocks = (int)((S + QB - 1) / QB);
  // One block fits per compute unit, so the grid runs in rounds of 256 blocks.  Whole rounds keep one
  // block per work id; the work ids left over for the last round are cut into key ranges (at least 8
  // key tiles each) so that the round is both shorter and wider, and a merge kernel joins the ranges.
  const int W = qblocks * h, NKT = (int)((L + 63) / 64);
  const int n_full = W / 256 * 256, n_tail = W - n_full;
  int parts = 1;
  if (n_tail > 0 && scratch) {
    parts = 256 / n_tail;
    if (parts > 8) parts = 8;
    if (parts > NKT / 8) parts = NKT / 8;
    if (parts < 1) parts = 1;
  }
  dim3 grid((unsigned)(n_full + (n_tail * parts + 7) / 8 * 8));
  static std::atomic<uint64_t> done;
  allow_dynamic_lds((const void*)k_attn_bf16<HD, QG, KG>, lds, done);
  k_attn_bf16<HD, QG, KG><<<grid, 512, lds, st>>>(q, q_head_stride, k, k_head_stride, k_row0, vt, vt_row_stride, S, L, out, ldo, qblocks, n_full, n_tail, parts, scratch, qn);
  if (parts > 1) {
    constexpr int QPB = 256 / (HD / 4);                  // queries per merge block
    k_attn_merge<HD, QB><<<(unsigned)(n_tail * (QB / QPB)), 256, 0, st>>>(scratch, n_full, n_tail, parts, qblocks, S, out, ldo);
  }
}

void launch_attn_bf16(const bf16_t* q, int64_t q_head_stride, const bf16_t* k, int64_t k_head_stride,
                      int64_t k_row0, const bf16_t* vt, int64_t vt_row_stride, int64_t S, int64_t L,
                      int h, int d, bf16_t* out, int64_t ldo, float* scratch, const AttnQNorm* qnorm, hipStream_t st) {
  if (S <= 0 || L <= 0) return;
  const AttnQNorm qn = qnorm ? *qnorm : AttnQNorm{nullptr, 0, 0, 0.f, 0.f, 0.f};
  // 256 queries per block share every K / V^T tile (half the LDS fill traffic per query) whenever that
  // still gives the grid half a round of blocks and the key range a few tiles; otherwise 128 queries per
  // block with the keys split over two groups, which halves the length of a block.
  const bool wide = L >= 256 && ((S + 255) / 256) * h >= 128;
#define ATTN_ARGS q, q_head_stride, k, k_head_stride, k_row0, vt, vt_row_stride, S, L, h, out, ldo, scratch, qn, st
  if (d == 128) { if (wide) launch_attn_cfg<128, 8, 1>(ATTN_ARGS); else launch_attn_cfg<128, 4, 2>(ATTN_ARGS); }
  else { if (wide) launch_attn_cfg<64, 8, 1>(ATTN_ARGS); else launch_attn_cfg<64, 4, 2>(ATTN_ARGS); }
#undef ATTN_ARGS
}
