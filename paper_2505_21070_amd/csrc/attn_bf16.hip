// Flash attention on the gfx950 matrix cores for the DP_BF16 path: the block's queries attend over one
// contiguous key range [cached prefix ; current block] streamed from HBM through LDS tiles, with an
// online softmax in fp32.  Used for self-attention (cache + block) and cross-attention (text keys).
//
// The scores are computed transposed, S^T = K * Q^T (keys are MFMA rows, queries MFMA columns): a
// lane then owns one query column, so the softmax max/sum are reductions over the lane's own
// registers plus one exchange with lane ^ 32, and the fp32 S^T accumulators, once exponentiated and
// rounded to bf16, ARE the B operand of the second product O^T = V^T * P^T (the k index of that
// product is a fixed permutation of the keys, applied to V^T when it is written to LDS).
//
// Block: 4 wavefronts x (QT x 32) queries of one head; key tile 64; K tile [64][HD] and V^T tile
// [HD][64] double-buffered in LDS; global loads for tile i+1 are in flight while tile i is used.
#include "kernels.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t cvt_pk_bf16(float a, float b) {
  f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

template <int HD, int QT>
__global__ __launch_bounds__(256) void k_attn_bf16(const bf16_t* __restrict__ q, int64_t q_head_stride,
                                                  const bf16_t* __restrict__ k, int64_t k_head_stride,
                                                  int64_t k_row0, const bf16_t* __restrict__ vt,
                                                  int64_t vt_row_stride, int64_t S, int64_t L,
                                                  bf16_t* __restrict__ out, int64_t ldo, float sc2) {
  constexpr int CR = HD / 8;                 // 16-byte chunks per K row
  constexpr int KS = HD / 16;                // MFMA k-steps over the head dim
  constexpr int DT = HD / 32;                // 32-row tiles of O^T
  constexpr int KCH = 64 * CR;               // chunks in the K tile
  constexpr int VCH = HD * 8;                // chunks in the V^T tile
  constexpr int STAGE = KCH + VCH;
  constexpr int CK = KCH / 256, CV = VCH / 256;
  __shared__ uint4 smem[2 * STAGE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lg = lane >> 5;
  const int head = blockIdx.y;
  const int64_t q0 = ((int64_t)blockIdx.x * 4 + wave) * (QT * 32);

  // Q fragments stay in registers: B operand, column = query, 8 head-dim values per lane
  bf16x8 qf[QT][KS];
  {
    const bf16_t* qh = q + (int64_t)head * q_head_stride;
#pragma unroll
    for (int t = 0; t < QT; ++t)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        qf[t][ks] = __builtin_bit_cast(bf16x8, *(const uint4*)(qh + (q0 + t * 32 + lr) * HD + ks * 16 + lg * 8));
  }
  const bf16_t* kh = k + (int64_t)head * k_head_stride + k_row0 * HD;
  const bf16_t* vh = vt + (int64_t)head * HD * vt_row_stride + k_row0;

  // global -> LDS assignment
  const uint4* gk[CK]; int sk[CK];
#pragma unroll
  for (int i = 0; i < CK; ++i) {
    const int c = tid + i * 256, row = c / CR, ch = c % CR;
    gk[i] = (const uint4*)(kh + (int64_t)row * HD + ch * 8);
    sk[i] = row * CR + (ch ^ (row & (CR - 1)));
  }
  const uint4* gv[CV]; int sv0[CV], sv1[CV];
#pragma unroll
  for (int i = 0; i < CV; ++i) {
    const int c = tid + i * 256, row = c >> 3, ch = c & 7;       // ch: 8 keys [8ch, 8ch+8)
    gv[i] = (const uint4*)(vh + (int64_t)row * vt_row_stride + ch * 8);
    // keys 8ch+0..3 -> chunk 2*(ch/2), half (ch&1); keys 8ch+4..7 -> chunk 2*(ch/2)+1, half (ch&1)
    const int c0 = (ch & ~1), c1 = c0 + 1;
    sv0[i] = (KCH + row * 8 + (c0 ^ (row & 7))) * 2 + (ch & 1);  // in 8-byte units
    sv1[i] = (KCH + row * 8 + (c1 ^ (row & 7))) * 2 + (ch & 1);
  }

  f32x16 oacc[DT][QT];
#pragma unroll
  for (int a = 0; a < DT; ++a)
#pragma unroll
    for (int t = 0; t < QT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[a][t][r] = 0.f;
  float mrun[QT], lsum[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) { mrun[t] = -INFINITY; lsum[t] = 0.f; }

  const int NKT = (int)((L + 63) / 64);
  uint4 rk[CK], rv[CV];
#pragma unroll
  for (int i = 0; i < CK; ++i) rk[i] = gk[i][0];
#pragma unroll
  for (int i = 0; i < CV; ++i) rv[i] = gv[i][0];
  {
    uint2* s2 = (uint2*)smem;
#pragma unroll
    for (int i = 0; i < CK; ++i) smem[sk[i]] = rk[i];
#pragma unroll
    for (int i = 0; i < CV; ++i) { s2[sv0[i]] = make_uint2(rv[i].x, rv[i].y); s2[sv1[i]] = make_uint2(rv[i].z, rv[i].w); }
  }
  __syncthreads();

  for (int kt = 0; kt < NKT; ++kt) {
    // prefetch the next key tile (the last iteration re-reads its own tile; the copy is never used)
    const int ktn = kt + 1 < NKT ? kt + 1 : kt;
#pragma unroll
    for (int i = 0; i < CK; ++i) rk[i] = gk[i][(int64_t)ktn * 64 * CR];            // 64 rows of CR chunks
#pragma unroll
    for (int i = 0; i < CV; ++i) rv[i] = gv[i][ktn * 8];                           // 64 keys = 8 chunks
    const uint4* buf = smem + (kt & 1) * STAGE;

    // S^T tiles: [2 key tiles of 32][QT query tiles]
    f32x16 sacc[2][QT];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int t = 0; t < QT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[a][t][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        const int row = a * 32 + lr, ch = ks * 2 + lg;
        const bf16x8 kf = __builtin_bit_cast(bf16x8, buf[row * CR + (ch ^ (row & (CR - 1)))]);
#pragma unroll
        for (int t = 0; t < QT; ++t)
          sacc[a][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t][ks], sacc[a][t], 0, 0, 0);
      }
    }
    // mask keys beyond L (last tile only): register r of tile a is key a*32 + (r/4)*8 + lg*4 + (r%4)
    const int kvalid = (int)(L - (int64_t)kt * 64);
    if (kvalid < 64) {
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = a * 32 + (r >> 2) * 8 + lg * 4 + (r & 3);
          if (key >= kvalid) {
#pragma unroll
            for (int t = 0; t < QT; ++t) sacc[a][t][r] = -INFINITY;
          }
        }
    }
    // online softmax per query column; probabilities packed as the B operand of O^T += V^T P^T
    uint4 pf[QT][4];
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      float mx = sacc[0][t][0];
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[a][t][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float mnew = fmaxf(mrun[t], mx * sc2);
      const float alpha = __builtin_amdgcn_exp2f(mrun[t] - mnew);
      mrun[t] = mnew;
      float ps = 0.f;
#pragma unroll
      for (int a = 0; a < 2; ++a) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          float p[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            p[j] = __builtin_amdgcn_exp2f(fmaf(sacc[a][t][u * 8 + j], sc2, -mnew));
            ps += p[j];
          }
          pf[t][a * 2 + u] = make_uint4(cvt_pk_bf16(p[0], p[1]), cvt_pk_bf16(p[2], p[3]),
                                        cvt_pk_bf16(p[4], p[5]), cvt_pk_bf16(p[6], p[7]));
        }
      }
      lsum[t] = lsum[t] * alpha + ps;
#pragma unroll
      for (int a = 0; a < DT; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[a][t][r] *= alpha;
    }
    // O^T += V^T * P^T
#pragma unroll
    for (int u4 = 0; u4 < 4; ++u4) {
#pragma unroll
      for (int a = 0; a < DT; ++a) {
        const int row = a * 32 + lr, ch = u4 * 2 + lg;
        const bf16x8 vf = __builtin_bit_cast(bf16x8, buf[KCH + row * 8 + (ch ^ (row & 7))]);
#pragma unroll
        for (int t = 0; t < QT; ++t)
          oacc[a][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, __builtin_bit_cast(bf16x8, pf[t][u4]), oacc[a][t], 0, 0, 0);
      }
    }
    {
      uint4* nb = smem + ((kt + 1) & 1) * STAGE;
      uint2* n2 = (uint2*)nb;
#pragma unroll
      for (int i = 0; i < CK; ++i) nb[sk[i]] = rk[i];
#pragma unroll
      for (int i = 0; i < CV; ++i) { n2[sv0[i]] = make_uint2(rv[i].x, rv[i].y); n2[sv1[i]] = make_uint2(rv[i].z, rv[i].w); }
    }
    __syncthreads();
  }

  // O[q][head*HD + c] = O^T[c][q] / l ; lane holds 4 consecutive c per register quad
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int64_t qi = q0 + t * 32 + lr;
    const float l = lsum[t] + __shfl_xor(lsum[t], 32, 64);
    const float inv = 1.f / l;
    if (qi < S) {
      bf16_t* o = out + qi * ldo + (int64_t)head * HD;
#pragma unroll
      for (int a = 0; a < DT; ++a)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int c = a * 32 + g4 * 8 + lg * 4;
          uint2 pk;
          pk.x = cvt_pk_bf16(oacc[a][t][g4 * 4 + 0] * inv, oacc[a][t][g4 * 4 + 1] * inv);
          pk.y = cvt_pk_bf16(oacc[a][t][g4 * 4 + 2] * inv, oacc[a][t][g4 * 4 + 3] * inv);
          *(uint2*)(o + c) = pk;
        }
    }
  }
}

void launch_attn_bf16(const bf16_t* q, int64_t q_head_stride, const bf16_t* k, int64_t k_head_stride,
                      int64_t k_row0, const bf16_t* vt, int64_t vt_row_stride, int64_t S, int64_t L,
                      int h, int d, bf16_t* out, int64_t ldo, hipStream_t st) {
  if (S <= 0 || L <= 0) return;
  const float sc2 = 1.4426950408889634f / sqrtf((float)d);
  constexpr int QT = 2;
  dim3 grid((unsigned)((S + 4 * QT * 32 - 1) / (4 * QT * 32)), (unsigned)h);
  if (d == 128)
    k_attn_bf16<128, QT><<<grid, 256, 0, st>>>(q, q_head_stride, k, k_head_stride, k_row0, vt, vt_row_stride, S, L, out, ldo, sc2);
  else
    k_attn_bf16<64, QT><<<grid, 256, 0, st>>>(q, q_head_stride, k, k_head_stride, k_row0, vt, vt_row_stride, S, L, out, ldo, sc2);
}
