// Host-side launchers of libdualparal's kernels.  Every launcher only enqueues work on `st`.
#pragma once
#include <atomic>
#include "common.h"

// ---- elementwise.hip -------------------------------------------------------------------------
template <typename T> void launch_to_f32(const T* in, float* out, int64_t n, hipStream_t st);
template <typename T> void launch_from_f32(const float* in, T* out, int64_t n, hipStream_t st);
// out[s,:] = LayerNorm(x[s,:]) * (mul + plus_one) + add ; x fp32 [S,D], mul/add fp32 [D].
// xin != null: the rows are read from xin (bf16 [S,D]) instead, and x receives their fp32 copy.
template <typename T>
void launch_ln_modulate(float* x, const bf16_t* xin, T* out, int64_t S, int D, float eps, const float* mul,
                        const float* add, int plus_one, hipStream_t st);

// src[S, ld] holds un-normalised projections; job j takes columns [col, col+D) of every row:
// dst[head][row0 + s][d] = out_scale * RoPE(RMSNorm_D(src[s, col:col+D]) * g) ; rope == 0 skips the rotation.
// Up to two jobs (e.g. q and k of the fused QKV output) run in one launch.  D % 8 == 0.
template <typename T> struct NormRopeJob {
  int col; const float* g; float out_scale; T* dst; int64_t head_stride; int64_t row0; int rope;
};
template <typename T>
void launch_norm_rope(const T* src, int64_t ld, int64_t S, int h, int d, float eps, const NormRopeJob<T>* jobs,
                      int n_jobs, const RopeTables* rope, int frame0, int tok_h, int tok_w, hipStream_t st);
// cs[s][i] = rotation (cos, sin) of channel pair i < head_dim / 2 at token s of a block that starts at frame0
void launch_rope_tokens(const RopeTables& rt, int frame0, int tok_h, int tok_w, int64_t S, float2* cs, hipStream_t st);
// k[head][row0 + s][:] *= rsqrt(sum_i ssq[i * stride + s] / (h * d) + eps), bf16 rows of d elements, in place
void launch_scale_rows_bf16(bf16_t* k, int64_t head_stride, int64_t row0, int64_t S, int h, int d, const float* ssq,
                            int np, int64_t stride, float eps, hipStream_t st);
// vt[head][c][col0 + s] = src[s, col + head*d + c]
template <typename T>
void launch_v_transpose(const T* src, int64_t ld, int col, int64_t S, int h, int d, T* vt,
                        int64_t row_stride, int64_t col0, hipStream_t st);
// dst[r][0..len) = src[r][0..len) for r < rows (strides in elements)
template <typename T>
void launch_copy2d(const T* src, int64_t src_stride, T* dst, int64_t dst_stride, int64_t rows,
                   int64_t len, hipStream_t st);
// out[n, k] = in[k, n] for n < N, zero rows for N <= n < Npad     (in [K, N] row-major)
template <typename T>
void launch_transpose_pad(const T* in, int64_t K, int64_t N, T* out, int64_t Npad, hipStream_t st);

void launch_sinusoid(float t, int freq_dim, float* out, hipStream_t st);
// Timestep-MLP matrix-vector product over sliced vectors.  A sliced vector is `parts` partial vectors
// (stride apart) whose sum, plus a bias, is the value.  y receives gemv_slices(K, N) <= GEMV_MAX_SLICES partial
// results [slice][N] of sum_k act(x[k]) * W[k, n], x[k] = sum_p x[p][k] + xbias[k]; act = SiLU when silu_in.
constexpr int GEMV_MAX_SLICES = 8;
int gemv_slices(int K, int N);
template <typename T>
void launch_gemv(const float* x, int x_parts, int x_stride, const T* xbias, int K, const T* W, int N, int silu_in,
                 float* y, hipStream_t st);
// mod[l, i] = mtab[l, i] + sum_p e[p][i] + bias[i]
template <typename T>
void launch_mod_add(const float* mtab, const float* e, int parts, const T* bias, float* mod, int L, int n, hipStream_t st);
void launch_rope_table(float2* tab, int n_pos, int pairs, float theta, hipStream_t st);
void launch_fill_zero(void* p, size_t bytes, hipStream_t st);
// dst[s, head*d + c] (fp32) = src[head][row0 + s][c]
template <typename T>
void launch_gather_heads(const T* src, int64_t head_stride, int64_t row0, int64_t S, int h, int d,
                         float* dst, hipStream_t st);
// dst[s, head*d + c] (fp32) = vt[head][c][col0 + s]
template <typename T>
void launch_gather_vt(const T* vt, int64_t row_stride, int64_t col0, int64_t S, int h, int d,
                      float* dst, hipStream_t st);

// ---- gemm_f32.hip : C = A[M,K] * W[K,N] (+ epilogue), all row-major, fp32 FMA ---------------
void launch_gemm_f32(const float* A, int64_t lda, const float* W, int64_t ldw, int64_t M, int64_t N,
                     int64_t K, int epi, const EpiArgs& e, hipStream_t st);
// ---- attn_f32.hip ----------------------------------------------------------------------------
// q [h][*][d] rows q_row0.., k [h][*][d] rows k_row0.. (L rows), vt [h][d][*] cols k_row0.. ;
// out[s, head*d + c], row stride ldo
void launch_attn_f32(const float* q, int64_t q_head_stride, const float* k, int64_t k_head_stride,
                     int64_t k_row0, const float* vt, int64_t vt_row_stride, int64_t S, int64_t L,
                     int h, int d, float* out, int64_t ldo, hipStream_t st);

// out[f, :] = pool[index[f], :], frame_bytes % 16 == 0, all pointers 16-byte aligned
void launch_gather_frames(const void* pool, int pool_frames, int64_t frame_bytes, const int32_t* index,
                          int n_frames, void* out, hipStream_t st);
// Raises a kernel's dynamic-LDS limit once per device and process (the attribute belongs to the device's copy
// of the code object).  `done` is one bit per device ordinal; safe to call from several host threads.
inline void allow_dynamic_lds(const void* kernel, int bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  (void)hipGetDevice(&dev);
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return;
  (void)hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  done.fetch_or(bit, std::memory_order_release);
}

// ---- gemm_bf16.hip : C = A[M,K] * Wt[N,K]^T (+ epilogue), bf16 MFMA, fp32 accumulate --------
// A must be readable for roundup(M, 256) rows, Wt for roundup(N, 256) rows; K % 64 == 0.
bool launch_gemm_bf16(const bf16_t* A, int64_t lda, const bf16_t* Wt, int64_t ldw, int64_t M,
                      int64_t N, int64_t K, int epi, const EpiArgs& e, hipStream_t st);
// whether launch_gemm_bf16(.., EPI_HEADS, ..) can take this problem; if not it launches nothing and returns false
bool gemm_bf16_heads_ok(int64_t M, int64_t N, const HeadsArgs& h);
// ---- attn_bf16.hip : flash attention on MFMA, head_dim 64 or 128 ------------------------------
// q must already be multiplied by log2(e)/sqrt(d) (attn_bf16_q_scale) and be readable for
// roundup(S, 256) rows per head; k rows / vt columns readable (finite in vt) up to
// k_row0 + roundup(L, 64).
// scratch: attn_bf16_scratch_bytes(d) bytes of device memory for the partial results of work that is
// split over key ranges (contents need not be kept between calls), or nullptr to never split.
inline float attn_bf16_q_scale(int d) { return 1.4426950408889634f / sqrtf((float)d); }
// Deferred RMSNorm of the queries: row s of q (all heads) is multiplied by
// rsqrt(sum_i ssq[i * stride + s] * inv_dim + eps) * scale as it is loaded (ssq == nullptr: q is used as stored).
struct AttnQNorm { const float* ssq; int np; int64_t stride; float inv_dim, eps, scale; };
// test hook: q[head][s][:] of all heads, token-major fp32, scaled and rounded exactly as the attention kernel does
void launch_gather_heads_qnorm(const bf16_t* src, int64_t head_stride, int64_t S, int h, int d, const AttnQNorm& qn,
                               float* dst, hipStream_t st);
// out[i] = a[i] * b[i]
void launch_mul_f32(const float* a, const float* b, float* out, int64_t n, hipStream_t st);
size_t attn_bf16_scratch_bytes(int d);
void launch_attn_bf16(const bf16_t* q, int64_t q_head_stride, const bf16_t* k, int64_t k_head_stride,
                      int64_t k_row0, const bf16_t* vt, int64_t vt_row_stride, int64_t S, int64_t L,
                      int h, int d, bf16_t* out, int64_t ldo, float* scratch, const AttnQNorm* qnorm, hipStream_t st);
