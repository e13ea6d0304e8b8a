// C-ABI of libdualparal: workspace layout, stage set-up, the per-block forward pass, the feature-cache
// hand-over and the test hook.  Every step of the pass is one of the library's own kernels; this file
// only orders them on the caller's stream.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/dualparal.h"
#include "kernels.h"

// ------------------------------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";
static int fail(int code, const char* fmt, ...) {
  va_list ap; va_start(ap, fmt); vsnprintf(g_err, sizeof(g_err), fmt, ap); va_end(ap);
  return code;
}
extern "C" const char* dp_last_error(void) { return g_err; }
// shared with schedule.cpp
int dp_set_error(int code, const char* msg) { return fail(code, "%s", msg); }

static inline int64_t rup(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

// ------------------------------------------------------------------------------------------ noise gather
extern "C" int dp_noise_gather(const void* pool, int32_t pool_frames, int64_t frame_bytes, const int32_t* index,
                               int32_t n_frames, void* out, void* hip_stream) {
  if (pool_frames < 1 || n_frames < 0 || frame_bytes < 0) return fail(DP_EINVAL, "dp_noise_gather: negative size");
  if (n_frames == 0 || frame_bytes == 0) return DP_OK;                  // nothing to copy
  if (!pool || !index || !out) return fail(DP_EINVAL, "dp_noise_gather: null pointer");
  if (frame_bytes % 16 || ((uintptr_t)pool & 15) || ((uintptr_t)out & 15))
    return fail(DP_EINVAL, "dp_noise_gather: frames must be multiples of 16 bytes and 16-byte aligned");
  if (n_frames > 65535) return fail(DP_EINVAL, "dp_noise_gather: more than 65535 frames in one call");
  launch_gather_frames(pool, pool_frames, frame_bytes, index, n_frames, out, (hipStream_t)hip_stream);
  return DP_OK;
}

// ------------------------------------------------------------------------------------------ layout
struct LayerMem {
  float *gq, *gk, *cgq, *cgk, *ln3g, *ln3b;     // fp32 copies of the per-channel vectors
  void *kbuf, *vtbuf;                           // [h][Lpad][d], [h][d][Lpad]: rows / columns = key positions of the buffer
  void *tk, *tvt;                               // text keys [h][Ltpad][d], text values transposed [h][d][Ltpad]
  void *tkq; float* cgqk;                       // heads_epi: text keys times the cross-attention query gains, and the gain product
  void *wqkv_t, *bqkv, *wo_t, *cwq_t, *cwo_t, *w1_t, *w2_t;   // bf16 path: weights as [out(pad 256), in]
};

struct Profiler {
  uint32_t mask = 0;
  std::vector<hipEvent_t> ev;     // pairs: (before, after)
  std::vector<int> cls;
  size_t used = 0;
  bool on(int c) const { return (mask >> c) & 1u; }
  bool begin(int c, hipStream_t st) {
    if (!on(c) || used + 2 > ev.size()) return false;
    (void)hipEventRecord(ev[used], st);
    return true;
  }
  void end(int c, hipStream_t st) {
    (void)hipEventRecord(ev[used + 1], st);
    cls.push_back(c);
    used += 2;
  }
  ~Profiler() { for (hipEvent_t e : ev) (void)hipEventDestroy(e); }
};
// times the launches in the statement block when class `c` is being profiled
#define PROF(c, ...) do { const bool _p = s->prof.begin((c), st); __VA_ARGS__; if (_p) s->prof.end((c), st); } while (0)

struct dp_stage {
  Profiler prof;
  dp_stage_config cfg;
  dp_stage_weights w;
  std::vector<dp_layer_weights> lw;
  std::vector<LayerMem> lm;
  int64_t tok, Smax, Ncmax, Spad, Lfit, Lpad, Ltpad, esz;
  // shared activations
  float* xres; void* hbuf; void* raw; void* qbuf; void* attn_o; void* mid;
  void* textpad; void* ctx; void* ctx_mid; void* wtmp;
  float *tau, *e1, *e2, *e0, *mtab, *mod;
  float2 *rope_f, *rope_y, *rope_x; RopeTables rt;
  void* tap_attn; float *tap_xself, *tap_xcross;
  float* attn_scratch;
  // DP_BF16 with dim % 256 == 0: the q/k/v and cross-q projections write per head from their GEMM epilogues
  // (gains and rotation applied there), leaving only the RMSNorm row scale, which arrives as partial sums
  float *qssq, *kssq; float2* rope_tok; int ssq_np, cross_np = 0; bool heads_epi; bool launch_ok = true;
  // state
  // Key buffer geometry (rows of kbuf = columns of vtbuf, the same in every layer).  The last block's keys
  // sit at [blk0, blk0 + last_S); the feature cache is the range [cache0, cache0 + cache_len): the sub-range
  // of the last block that dp_cache_update named, left where it is whenever a maximal block still fits on one
  // side of it, else a copy of it in the free space beside the last block.  The next block is written directly
  // before or directly after the cache, so the keys an attention call reads are always one contiguous range.
  int64_t blk0 = 0, cache0 = 0, cache_len = 0, last_S = 0; int last_frames = 0;
};

struct Carver {
  char* base; size_t off = 0;
  explicit Carver(void* b) : base((char*)b) {}
  void* take(size_t bytes) {
    off = (size_t)rup((int64_t)off, 256);
    void* p = base ? base + off : nullptr;
    off += bytes;
    return p;
  }
};

static const char* validate(const dp_stage_config* c) {
  if (!c) return "null config";
  if (c->n_layers < 1 || c->dim < 1 || c->n_heads < 1 || c->ffn_dim < 1) return "non-positive size";
  if ((int64_t)c->n_heads * c->head_dim != c->dim) return "n_heads * head_dim != dim";
  if (c->head_dim != 64 && c->head_dim != 128) return "head_dim must be 64 or 128";
  if (c->dim % 8 != 0 || c->dim > 8192) return "dim must be a multiple of 8 and at most 8192";
  if (c->text_len < 1 || c->text_dim < 1) return "text_len / text_dim must be positive";
  if (c->tok_h < 1 || c->tok_w < 1) return "tok_h / tok_w must be positive";
  if (c->max_block_frames < 1 || c->max_cache_frames < 0 || c->max_abs_frames < c->max_block_frames)
    return "bad frame limits";
  if (c->dtype != DP_F32 && c->dtype != DP_BF16) return "dtype must be DP_F32 or DP_BF16";
  if (c->freq_dim < 2 || (c->freq_dim & 1)) return "freq_dim must be even";
  if (!(c->rope_theta > 0.f) || !(c->eps >= 0.f)) return "bad rope_theta / eps";
  // Upper limits far beyond any model, so that no size below can overflow 64 bits or a 32-bit grid:
  // 2^24 tokens per block and in the cache, 2^24 frame positions, 2^20 text tokens
  if (c->n_layers > 1024 || c->ffn_dim > (1 << 17) || c->text_dim > (1 << 16) || c->text_len > (1 << 20) ||
      c->freq_dim > (1 << 16) || c->max_abs_frames > (1 << 24))
    return "n_layers / ffn_dim / text_dim / text_len / freq_dim / max_abs_frames beyond the supported range";
  if ((int64_t)c->tok_h * c->tok_w > (1 << 24) || (int64_t)c->tok_h * c->tok_w * c->max_block_frames > (1 << 24) ||
      (int64_t)c->tok_h * c->tok_w * c->max_cache_frames > (1 << 24))
    return "more than 2^24 tokens in a block or in the cache";
  {
    const int64_t spad = rup((int64_t)c->tok_h * c->tok_w * c->max_block_frames, 256);
    if (rup(c->text_len, 256) > 3 * spad) return "text_len too large for the block size";
  }
  if (c->weight_layout != DP_WEIGHTS_IN_OUT && c->weight_layout != DP_WEIGHTS_OUT_IN) return "unknown weight_layout";
  if (c->weight_layout == DP_WEIGHTS_OUT_IN) {
    // the GEMM tiles read whole groups of 256 weight rows: in the caller's memory there is no padding to read
    if (c->dtype != DP_BF16) return "DP_WEIGHTS_OUT_IN is a layout of the bf16 path";
    if (c->dim % 256 || c->ffn_dim % 256) return "DP_WEIGHTS_OUT_IN needs dim and ffn_dim % 256 == 0";
  }
  if (c->dtype == DP_BF16) {
    if (c->dim % 64 || c->ffn_dim % 64 || c->text_dim % 64) return "bf16 path needs dim, ffn_dim, text_dim % 64 == 0";
    if (((int64_t)c->tok_h * c->tok_w) % 8) return "bf16 path needs tok_h * tok_w % 8 == 0";
  }
  return nullptr;
}

// Lays the workspace out.  With base == nullptr it only measures.
static size_t carve(dp_stage* s, void* base) {
  const dp_stage_config& c = s->cfg;
  const bool bf = c.dtype == DP_BF16;
  s->esz = bf ? 2 : 4;
  s->tok = (int64_t)c.tok_h * c.tok_w;
  s->Smax = s->tok * c.max_block_frames;
  s->Ncmax = s->tok * c.max_cache_frames;
  s->Spad = rup(s->Smax, 256);
  // Key positions per layer: Num_B + Num_C frames when the block limit is Num_B and the cache limit Num_C / 2,
  // the live K/V of the paper's memory analysis (Table 1).  dp_cache_update keeps the retained range where a
  // maximal block fits on one side of it (see there); + one 64-key tile of padding for the attention loads.
  s->Lfit = s->Smax + 2 * s->Ncmax;
  s->Lpad = rup(s->Lfit, 64) + 64;
  s->Ltpad = rup(c.text_len, 256);
  const int64_t D = c.dim, F = c.ffn_dim, E = s->esz, L = c.n_layers;
  Carver cv(base);
  s->xres = (float*)cv.take(s->Spad * D * 4);
  s->hbuf = cv.take(s->Spad * D * E);
  s->raw = cv.take(s->Spad * 3 * D * E);
  s->qbuf = cv.take(s->Spad * D * E);
  s->attn_o = cv.take(s->Spad * D * E);
  s->mid = cv.take(s->Spad * F * E);
  s->textpad = cv.take(s->Ltpad * c.text_dim * E);
  s->ctx = cv.take(s->Ltpad * D * E);
  s->ctx_mid = cv.take(s->Ltpad * D * E);
  const int64_t kmax = c.text_dim > D ? c.text_dim : D;
  const bool own = bf && c.weight_layout == DP_WEIGHTS_IN_OUT;   // the library keeps [out, in] copies of the matrices
  s->wtmp = own ? cv.take(rup(D, 256) * kmax * E) : nullptr;
  s->heads_epi = bf && D % 256 == 0;
  s->ssq_np = (int)(D / 128);                         // most partial sums per row any tile shape produces
  s->qssq = s->heads_epi ? (float*)cv.take(s->Smax * s->ssq_np * 4) : nullptr;
  s->kssq = s->heads_epi ? (float*)cv.take(s->Smax * s->ssq_np * 4) : nullptr;
  s->rope_tok = s->heads_epi ? (float2*)cv.take(s->Smax * (c.head_dim / 2) * 8) : nullptr;
  s->tau = (float*)cv.take(c.freq_dim * 4);
  s->e1 = (float*)cv.take(GEMV_MAX_SLICES * D * 4); s->e2 = (float*)cv.take(GEMV_MAX_SLICES * D * 4);   // sliced vectors
  s->e0 = (float*)cv.take(GEMV_MAX_SLICES * 6 * D * 4);
  s->mtab = (float*)cv.take(L * 6 * D * 4);
  s->mod = (float*)cv.take(L * 6 * D * 4);
  const int half = c.head_dim / 2, c_sp = c.head_dim / 6, c_f = half - 2 * c_sp;
  s->rope_f = (float2*)cv.take((size_t)c.max_abs_frames * c_f * 8);
  s->rope_y = (float2*)cv.take((size_t)c.tok_h * (c_sp > 0 ? c_sp : 1) * 8);
  s->rope_x = (float2*)cv.take((size_t)c.tok_w * (c_sp > 0 ? c_sp : 1) * 8);
  s->rt = RopeTables{s->rope_f, s->rope_y, s->rope_x, c_f, c_sp, c_sp};
  if (c.debug_taps) {
    s->tap_attn = cv.take(s->Spad * D * E);
    s->tap_xself = (float*)cv.take(s->Spad * D * 4);
    s->tap_xcross = (float*)cv.take(s->Spad * D * 4);
  } else { s->tap_attn = nullptr; s->tap_xself = s->tap_xcross = nullptr; }
  s->lm.assign((size_t)L, LayerMem{});
  for (int64_t l = 0; l < L; ++l) {
    LayerMem& m = s->lm[(size_t)l];
    m.gq = (float*)cv.take(D * 4); m.gk = (float*)cv.take(D * 4);
    m.cgq = (float*)cv.take(D * 4); m.cgk = (float*)cv.take(D * 4);
    m.ln3g = (float*)cv.take(D * 4); m.ln3b = (float*)cv.take(D * 4);
    m.kbuf = cv.take(s->Lpad * D * E); m.vtbuf = cv.take(s->Lpad * D * E);
    m.tk = cv.take(s->Ltpad * D * E);
    m.tkq = s->heads_epi ? cv.take(s->Ltpad * D * E) : nullptr;
    m.cgqk = s->heads_epi ? (float*)cv.take(D * 4) : nullptr;
    m.tvt = cv.take(s->Ltpad * D * E);
  }
  const size_t zero_end = cv.off;      // everything up to here is zero-filled at init
  s->attn_scratch = bf ? (float*)cv.take(attn_bf16_scratch_bytes(c.head_dim)) : nullptr;
  if (bf) {
    for (int64_t l = 0; l < L; ++l) {
      LayerMem& m = s->lm[(size_t)l];
      m.bqkv = cv.take(3 * D * E);
      if (!own) continue;                               // handed over as [out, in]: read in place (see init_typed)
      m.wqkv_t = cv.take(rup(3 * D, 256) * D * E);
      m.wo_t = cv.take(rup(D, 256) * D * E); m.cwq_t = cv.take(rup(D, 256) * D * E);
      m.cwo_t = cv.take(rup(D, 256) * D * E);
      m.w1_t = cv.take(rup(F, 256) * D * E); m.w2_t = cv.take(rup(D, 256) * F * E);
    }
  }
  (void)zero_end;
  return (size_t)rup((int64_t)cv.off, 256);
}

static size_t zero_span(dp_stage* s) {   // bytes from the workspace start that must start as zeros
  const LayerMem& m = s->lm.back();
  return (size_t)((char*)m.tvt - (char*)s->xres) + (size_t)(s->Ltpad * s->cfg.dim * s->esz);
}

extern "C" size_t dp_stage_workspace_bytes(const dp_stage_config* cfg) {
  const char* why = validate(cfg);
  if (why) { fail(DP_EINVAL, "dp_stage_workspace_bytes: %s", why); return 0; }
  try {
    dp_stage tmp; tmp.cfg = *cfg;
    return carve(&tmp, nullptr);
  } catch (const std::bad_alloc&) {
    fail(DP_ENOMEM, "dp_stage_workspace_bytes: out of host memory");
    return 0;
  }
}

// ------------------------------------------------------------------------------------------ typed helpers
template <typename T> struct Path;
template <> struct Path<float> {
  static float q_scale(int) { return 1.f; }             // the fp32 attention kernel scales by 1/sqrt(d) itself
  // y = x[M,K] * W[K,N] (+epilogue); `wt` unused
  static bool gemm(const void* A, int64_t lda, const void* W, const void* /*wt*/, int64_t M, int64_t N,
                   int64_t K, int epi, const EpiArgs& e, hipStream_t st) {
    launch_gemm_f32((const float*)A, lda, (const float*)W, N, M, N, K, epi, e, st);
    return true;
  }
  static void attn(const void* q, int64_t qhs, const void* k, int64_t khs, int64_t row0, const void* vt,
                   int64_t vrs, int64_t S, int64_t L, int h, int d, void* out, int64_t ldo, float* /*scratch*/,
                   const AttnQNorm* /*qn*/, hipStream_t st) {
    launch_attn_f32((const float*)q, qhs, (const float*)k, khs, row0, (const float*)vt, vrs, S, L, h, d, (float*)out, ldo, st);
  }
};
template <> struct Path<bf16_t> {
  static float q_scale(int d) { return attn_bf16_q_scale(d); }   // queries carry log2(e)/sqrt(d)
  static bool gemm(const void* A, int64_t lda, const void* /*W*/, const void* wt, int64_t M, int64_t N,
                   int64_t K, int epi, const EpiArgs& e, hipStream_t st) {
    return launch_gemm_bf16((const bf16_t*)A, lda, (const bf16_t*)wt, K, M, N, K, epi, e, st);
  }
  static void attn(const void* q, int64_t qhs, const void* k, int64_t khs, int64_t row0, const void* vt,
                   int64_t vrs, int64_t S, int64_t L, int h, int d, void* out, int64_t ldo, float* scratch,
                   const AttnQNorm* qn, hipStream_t st) {
    launch_attn_bf16((const bf16_t*)q, qhs, (const bf16_t*)k, khs, row0, (const bf16_t*)vt, vrs, S, L, h, d, (bf16_t*)out, ldo, scratch, qn, st);
  }
};

static EpiArgs epi_store(void* out, int64_t ldo, const void* bias) { return EpiArgs{out, ldo, bias, nullptr, 0, nullptr}; }
static EpiArgs epi_resid(float* resid, int64_t ldr, const void* bias, const float* gate) {
  return EpiArgs{nullptr, 0, bias, resid, ldr, gate};
}

// ------------------------------------------------------------------------------------------ init
template <typename T>
static void init_typed(dp_stage* s, const void* text, hipStream_t st) {
  const dp_stage_config& c = s->cfg;
  const int64_t D = c.dim, F = c.ffn_dim, Lt = c.text_len, Td = c.text_dim;
  const int h = c.n_heads, d = c.head_dim;
  constexpr bool bf = sizeof(T) == 2;
  const bool own = bf && c.weight_layout == DP_WEIGHTS_IN_OUT;
  launch_fill_zero(s->xres, zero_span(s), st);
  launch_rope_table(s->rope_f, c.max_abs_frames, s->rt.c_f, c.rope_theta, st);
  launch_rope_table(s->rope_y, c.tok_h, s->rt.c_h, c.rope_theta, st);
  launch_rope_table(s->rope_x, c.tok_w, s->rt.c_w, c.rope_theta, st);
  for (int l = 0; l < c.n_layers; ++l) {
    const dp_layer_weights& w = s->lw[(size_t)l]; LayerMem& m = s->lm[(size_t)l];
    launch_to_f32<T>((const T*)w.mod, s->mtab + (int64_t)l * 6 * D, 6 * D, st);
    launch_to_f32<T>((const T*)w.gq, m.gq, D, st); launch_to_f32<T>((const T*)w.gk, m.gk, D, st);
    launch_to_f32<T>((const T*)w.cgq, m.cgq, D, st); launch_to_f32<T>((const T*)w.cgk, m.cgk, D, st);
    launch_to_f32<T>((const T*)w.ln3_g, m.ln3g, D, st); launch_to_f32<T>((const T*)w.ln3_b, m.ln3b, D, st);
    if (bf) {
      launch_copy2d<T>((const T*)w.bq, 0, (T*)m.bqkv, 0, 1, D, st);
      launch_copy2d<T>((const T*)w.bk, 0, (T*)m.bqkv + D, 0, 1, D, st);
      launch_copy2d<T>((const T*)w.bv, 0, (T*)m.bqkv + 2 * D, 0, 1, D, st);
    }
    if (bf && !own) {
      // [out, in] already, q | k | v rows in one matrix (checked by dp_stage_init): the GEMMs read the caller's memory
      m.wqkv_t = (void*)w.wq; m.wo_t = (void*)w.wo; m.cwq_t = (void*)w.cwq; m.cwo_t = (void*)w.cwo;
      m.w1_t = (void*)w.w1; m.w2_t = (void*)w.w2;
    }
    if (own) {
      T* qkv = (T*)m.wqkv_t;
      launch_transpose_pad<T>((const T*)w.wq, D, D, qkv, D, st);
      launch_transpose_pad<T>((const T*)w.wk, D, D, qkv + D * D, D, st);
      launch_transpose_pad<T>((const T*)w.wv, D, D, qkv + 2 * D * D, rup(3 * D, 256) - 2 * D, st);
      launch_transpose_pad<T>((const T*)w.wo, D, D, (T*)m.wo_t, rup(D, 256), st);
      launch_transpose_pad<T>((const T*)w.cwq, D, D, (T*)m.cwq_t, rup(D, 256), st);
      launch_transpose_pad<T>((const T*)w.cwo, D, D, (T*)m.cwo_t, rup(D, 256), st);
      launch_transpose_pad<T>((const T*)w.w1, D, F, (T*)m.w1_t, rup(F, 256), st);
      launch_transpose_pad<T>((const T*)w.w2, F, D, (T*)m.w2_t, rup(D, 256), st);
    }
  }
  // text side, once per prompt: optional MLP text_dim -> dim -> dim (tanh-GELU between), then every
  // layer's cross-attention keys (RMSNorm, no rotation) and values
  launch_copy2d<T>((const T*)text, Td, (T*)s->textpad, Td, Lt, Td, st);
  const void* ctx = s->textpad;
  if (Td != D) {
    if (own) launch_transpose_pad<T>((const T*)s->w.wx1, Td, D, (T*)s->wtmp, rup(D, 256), st);
    Path<T>::gemm(s->textpad, Td, s->w.wx1, own ? s->wtmp : s->w.wx1, Lt, D, Td, EPI_GELU, epi_store(s->ctx_mid, D, s->w.bx1), st);
    if (own) launch_transpose_pad<T>((const T*)s->w.wx2, D, D, (T*)s->wtmp, rup(D, 256), st);
    Path<T>::gemm(s->ctx_mid, D, s->w.wx2, own ? s->wtmp : s->w.wx2, Lt, D, D, EPI_STORE, epi_store(s->ctx, D, s->w.bx2), st);
    ctx = s->ctx;
  }
  for (int l = 0; l < c.n_layers; ++l) {
    const dp_layer_weights& w = s->lw[(size_t)l]; LayerMem& m = s->lm[(size_t)l];
    if (own) launch_transpose_pad<T>((const T*)w.cwk, D, D, (T*)s->wtmp, rup(D, 256), st);
    Path<T>::gemm(ctx, D, w.cwk, own ? s->wtmp : w.cwk, Lt, D, D, EPI_STORE, epi_store(s->raw, D, w.cbk), st);
    { const NormRopeJob<T> jk{0, m.cgk, 1.f, (T*)m.tk, s->Ltpad * d, 0, 0};
      launch_norm_rope<T>((const T*)s->raw, D, Lt, h, d, c.eps, &jk, 1, nullptr, 0, 1, 1, st); }
    if (s->heads_epi) {
      // q.k with q = r (q_raw * cgq): the query gains move over to the keys, the row scale r to the attention kernel
      launch_mul_f32(m.cgk, m.cgq, m.cgqk, D, st);
      const NormRopeJob<T> jk{0, m.cgqk, 1.f, (T*)m.tkq, s->Ltpad * d, 0, 0};
      launch_norm_rope<T>((const T*)s->raw, D, Lt, h, d, c.eps, &jk, 1, nullptr, 0, 1, 1, st);
    }
    if (own) launch_transpose_pad<T>((const T*)w.cwv, D, D, (T*)s->wtmp, rup(D, 256), st);
    Path<T>::gemm(ctx, D, w.cwv, own ? s->wtmp : w.cwv, Lt, D, D, EPI_STORE, epi_store(s->raw, D, w.cbv), st);
    launch_v_transpose<T>((const T*)s->raw, D, 0, Lt, h, d, (T*)m.tvt, s->Ltpad, 0, st);
  }
}

extern "C" int dp_stage_init(const dp_stage_config* cfg, const dp_stage_weights* weights, const void* text,
                             void* workspace, size_t workspace_bytes, void* hip_stream, dp_stage_t** out) {
  if (!out) return fail(DP_EINVAL, "dp_stage_init: out is null");
  *out = nullptr;
  const char* why = validate(cfg);
  if (why) return fail(DP_EINVAL, "dp_stage_init: %s", why);
  if (!weights || !weights->layers || !text || !workspace) return fail(DP_EINVAL, "dp_stage_init: null pointer");
  if (((uintptr_t)workspace) % 256) return fail(DP_EINVAL, "dp_stage_init: workspace must be 256-byte aligned");
  if (!weights->wt1 || !weights->bt1 || !weights->wt2 || !weights->bt2 || !weights->wm || !weights->bm)
    return fail(DP_EINVAL, "dp_stage_init: null timestep-MLP weight");
  if (cfg->text_dim != cfg->dim && (!weights->wx1 || !weights->bx1 || !weights->wx2 || !weights->bx2))
    return fail(DP_EINVAL, "dp_stage_init: text_dim != dim needs the text MLP weights");
  for (int l = 0; l < cfg->n_layers; ++l) {
    const void* const* p = (const void* const*)&weights->layers[l];
    for (size_t i = 0; i < sizeof(dp_layer_weights) / sizeof(void*); ++i)
      if (!p[i]) return fail(DP_EINVAL, "dp_stage_init: layer %d has a null weight pointer (field %zu)", l, i);
  }
  if (cfg->weight_layout == DP_WEIGHTS_OUT_IN) {
    // read in place by 16-byte loads; q | k | v rows form the one matrix the fused projection multiplies by
    const size_t dd = (size_t)cfg->dim * cfg->dim * 2;
    auto misaligned = [](const void* p) { return ((uintptr_t)p & 15) != 0; };
    if (cfg->text_dim != cfg->dim && (misaligned(weights->wx1) || misaligned(weights->wx2)))
      return fail(DP_EINVAL, "dp_stage_init: DP_WEIGHTS_OUT_IN matrices must be 16-byte aligned");
    for (int l = 0; l < cfg->n_layers; ++l) {
      const dp_layer_weights& w = weights->layers[l];
      if ((const char*)w.wk != (const char*)w.wq + dd || (const char*)w.wv != (const char*)w.wq + 2 * dd)
        return fail(DP_EINVAL, "dp_stage_init: layer %d: DP_WEIGHTS_OUT_IN needs wq, wk, wv back to back in one "
                               "[3 * dim, dim] matrix", l);
      if (misaligned(w.wq) || misaligned(w.wo) || misaligned(w.cwq) || misaligned(w.cwk) || misaligned(w.cwv) ||
          misaligned(w.cwo) || misaligned(w.w1) || misaligned(w.w2))
        return fail(DP_EINVAL, "dp_stage_init: layer %d: DP_WEIGHTS_OUT_IN matrices must be 16-byte aligned", l);
    }
  }
  dp_stage* s = new (std::nothrow) dp_stage();
  if (!s) return fail(DP_ENOMEM, "dp_stage_init: host allocation failed");
  s->cfg = *cfg; s->w = *weights;
  size_t need = 0;
  try {
    s->lw.assign(weights->layers, weights->layers + cfg->n_layers);
    s->w.layers = s->lw.data();
    need = carve(s, nullptr);
  } catch (const std::bad_alloc&) {
    delete s;
    return fail(DP_ENOMEM, "dp_stage_init: host allocation failed");
  }
  if (workspace_bytes < need) {
    delete s;
    return fail(DP_ENOMEM, "dp_stage_init: workspace has %zu bytes, %zu needed", workspace_bytes, need);
  }
  carve(s, workspace);
  hipStream_t st = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  if (cfg->dtype == DP_BF16) init_typed<bf16_t>(s, text, st); else init_typed<float>(s, text, st);
  const hipError_t err = hipGetLastError();
  if (err != hipSuccess) { delete s; return fail(DP_EHIP, "dp_stage_init: %s", hipGetErrorString(err)); }
  *out = s;
  return DP_OK;
}

extern "C" void dp_stage_free(dp_stage_t* stage) { delete stage; }

// ------------------------------------------------------------------------------------------ forward
template <typename T>
static void forward_typed(dp_stage* s, const void* x_in, void* x_out, int n_frames, int frame0, float t, hipStream_t st) {
  const dp_stage_config& c = s->cfg;
  const int64_t D = c.dim, F = c.ffn_dim, S = s->tok * n_frames;
  const int h = c.n_heads, d = c.head_dim;
  constexpr bool bf = sizeof(T) == 2;
  // bf16 storage: the first LayerNorm reads x_in itself and leaves its fp32 copy in the residual stream, and
  // the last GEMM writes x_out next to its residual update, so neither end needs a conversion pass
  if (!bf) PROF(DP_PROF_CONVERT, launch_to_f32<T>((const T*)x_in, s->xres, S * D, st));
  // adaLN modulation: sinusoidal features -> two-layer MLP (SiLU) -> SiLU -> 6*dim head, plus each layer's table
  PROF(DP_PROF_MODULATION,
       launch_sinusoid(t, c.freq_dim, s->tau, st);
       launch_gemv<T>(s->tau, 1, 0, (const T*)nullptr, c.freq_dim, (const T*)s->w.wt1, (int)D, 0, s->e1, st);
       launch_gemv<T>(s->e1, gemv_slices(c.freq_dim, (int)D), (int)D, (const T*)s->w.bt1, (int)D, (const T*)s->w.wt2, (int)D, 1, s->e2, st);
       launch_gemv<T>(s->e2, gemv_slices((int)D, (int)D), (int)D, (const T*)s->w.bt2, (int)D, (const T*)s->w.wm, (int)(6 * D), 1, s->e0, st);
       launch_mod_add<T>(s->mtab, s->e0, gemv_slices((int)D, (int)(6 * D)), (const T*)s->w.bm, s->mod, c.n_layers, (int)(6 * D), st));
  const int64_t kv_hs = s->Lpad * d;        // head stride of kbuf
  // where this block's keys go: directly before the cached range if it fits there, else directly after it
  // (dp_cache_update left the cache where one side has room for a maximal block)
  int64_t blk0 = 0, key0 = 0;
  if (s->cache_len > 0) {
    if (s->cache0 >= S) { blk0 = s->cache0 - S; key0 = blk0; }
    else { blk0 = s->cache0 + s->cache_len; key0 = s->cache0; }
  }
  s->blk0 = blk0;
  if (s->heads_epi) PROF(DP_PROF_NORM_ROPE, launch_rope_tokens(s->rt, frame0, c.tok_h, c.tok_w, S, s->rope_tok, st));
  for (int l = 0; l < c.n_layers; ++l) {
    const dp_layer_weights& w = s->lw[(size_t)l]; LayerMem& m = s->lm[(size_t)l];
    const float* md = s->mod + (int64_t)l * 6 * D;
    const float *sh1 = md, *sc1 = md + D, *g1 = md + 2 * D, *sh2 = md + 3 * D, *sc2 = md + 4 * D, *g2 = md + 5 * D;
    // --- self-attention over [cached K/V ; this block]
    PROF(DP_PROF_LN, launch_ln_modulate<T>(s->xres, bf && l == 0 ? (const bf16_t*)x_in : nullptr, (T*)s->hbuf, S, (int)D,
                                           c.eps, sc1, sh1, 1, st));
    AttnQNorm qn{s->qssq, 0, s->Smax, 1.f / (float)D, c.eps, Path<T>::q_scale(d)};
    if (s->heads_epi) {
      HeadsArgs ha{};
      ha.dim = (int)D; ha.head_dim = d; ha.cs = s->rope_tok; ha.ssq_stride = s->Smax;
      ha.sec[0] = HeadSection{s->qbuf, s->Spad * d, 0, m.gq, s->qssq, 1, 0};
      ha.sec[1] = HeadSection{m.kbuf, kv_hs, blk0, m.gk, s->kssq, 1, 0};
      ha.sec[2] = HeadSection{m.vtbuf, s->Lpad, blk0, nullptr, nullptr, 0, 1};
      EpiArgs e = epi_store(nullptr, 0, m.bqkv);
      e.heads = &ha;
      PROF(DP_PROF_QKV_GEMM, s->launch_ok &= Path<T>::gemm(s->hbuf, D, nullptr, m.wqkv_t, S, 3 * D, D, EPI_HEADS, e, st));
      qn.np = ha.ssq_np;
      PROF(DP_PROF_NORM_ROPE, launch_scale_rows_bf16((bf16_t*)m.kbuf, kv_hs, blk0, S, h, d, s->kssq, ha.ssq_np, s->Smax, c.eps, st));
    } else {
      if (bf) {
        PROF(DP_PROF_QKV_GEMM,
             Path<T>::gemm(s->hbuf, D, nullptr, m.wqkv_t, S, 3 * D, D, EPI_STORE, epi_store(s->raw, 3 * D, m.bqkv), st));
      } else {
        PROF(DP_PROF_QKV_GEMM,
             Path<T>::gemm(s->hbuf, D, w.wq, nullptr, S, D, D, EPI_STORE, epi_store(s->raw, 3 * D, w.bq), st);
             Path<T>::gemm(s->hbuf, D, w.wk, nullptr, S, D, D, EPI_STORE, epi_store((T*)s->raw + D, 3 * D, w.bk), st);
             Path<T>::gemm(s->hbuf, D, w.wv, nullptr, S, D, D, EPI_STORE, epi_store((T*)s->raw + 2 * D, 3 * D, w.bv), st));
      }
      PROF(DP_PROF_NORM_ROPE,
           const NormRopeJob<T> qk[2] = {{0, m.gq, Path<T>::q_scale(d), (T*)s->qbuf, s->Spad * d, 0, 1},
                                         {(int)D, m.gk, 1.f, (T*)m.kbuf, kv_hs, blk0, 1}};
           launch_norm_rope<T>((const T*)s->raw, 3 * D, S, h, d, c.eps, qk, 2, &s->rt, frame0, c.tok_h, c.tok_w, st);
           launch_v_transpose<T>((const T*)s->raw, 3 * D, (int)(2 * D), S, h, d, (T*)m.vtbuf, s->Lpad, blk0, st));
    }
    PROF(DP_PROF_SELF_ATTN,
         Path<T>::attn(s->qbuf, s->Spad * d, m.kbuf, kv_hs, key0, m.vtbuf, s->Lpad, S,
                       s->cache_len + S, h, d, s->attn_o, D, s->attn_scratch, s->heads_epi ? &qn : nullptr, st));
    if (s->tap_attn && l == c.n_layers - 1) launch_copy2d<T>((const T*)s->attn_o, 0, (T*)s->tap_attn, 0, 1, S * D, st);
    PROF(DP_PROF_OPROJ_GEMM, Path<T>::gemm(s->attn_o, D, w.wo, m.wo_t, S, D, D, EPI_RESID, epi_resid(s->xres, D, w.bo, g1), st));
    if (s->tap_xself && l == c.n_layers - 1) launch_copy2d<float>(s->xres, 0, s->tap_xself, 0, 1, S * D, st);
    // --- cross-attention to the text tokens
    PROF(DP_PROF_LN, launch_ln_modulate<T>(s->xres, nullptr, (T*)s->hbuf, S, (int)D, c.eps, m.ln3g, m.ln3b, 0, st));
    if (s->heads_epi) {
      HeadsArgs ha{};
      ha.dim = (int)D; ha.head_dim = d; ha.ssq_stride = s->Smax;
      ha.sec[0] = HeadSection{s->qbuf, s->Spad * d, 0, nullptr, s->qssq, 0, 0};
      EpiArgs e = epi_store(nullptr, 0, w.cbq);
      e.heads = &ha;
      PROF(DP_PROF_CROSS_Q_GEMM, s->launch_ok &= Path<T>::gemm(s->hbuf, D, w.cwq, m.cwq_t, S, D, D, EPI_HEADS, e, st));
      qn.np = ha.ssq_np;
      s->cross_np = ha.ssq_np;
      PROF(DP_PROF_CROSS_ATTN,
           Path<T>::attn(s->qbuf, s->Spad * d, m.tkq, s->Ltpad * d, 0, m.tvt, s->Ltpad, S, c.text_len, h, d, s->attn_o, D, s->attn_scratch, &qn, st));
    } else {
      PROF(DP_PROF_CROSS_Q_GEMM, Path<T>::gemm(s->hbuf, D, w.cwq, m.cwq_t, S, D, D, EPI_STORE, epi_store(s->raw, D, w.cbq), st));
      PROF(DP_PROF_NORM_ROPE,
           const NormRopeJob<T> cq{0, m.cgq, Path<T>::q_scale(d), (T*)s->qbuf, s->Spad * d, 0, 0};
           launch_norm_rope<T>((const T*)s->raw, D, S, h, d, c.eps, &cq, 1, nullptr, 0, 1, 1, st));
      PROF(DP_PROF_CROSS_ATTN,
           Path<T>::attn(s->qbuf, s->Spad * d, m.tk, s->Ltpad * d, 0, m.tvt, s->Ltpad, S, c.text_len, h, d, s->attn_o, D, s->attn_scratch, nullptr, st));
    }
    PROF(DP_PROF_CROSS_O_GEMM, Path<T>::gemm(s->attn_o, D, w.cwo, m.cwo_t, S, D, D, EPI_RESID, epi_resid(s->xres, D, w.cbo, nullptr), st));
    if (s->tap_xcross && l == c.n_layers - 1) launch_copy2d<float>(s->xres, 0, s->tap_xcross, 0, 1, S * D, st);
    // --- FFN
    PROF(DP_PROF_LN, launch_ln_modulate<T>(s->xres, nullptr, (T*)s->hbuf, S, (int)D, c.eps, sc2, sh2, 1, st));
    PROF(DP_PROF_FFN1_GEMM, Path<T>::gemm(s->hbuf, D, w.w1, m.w1_t, S, F, D, EPI_GELU, epi_store(s->mid, F, w.b1), st));
    EpiArgs e2 = epi_resid(s->xres, D, w.b2, g2);
    if (bf && l == c.n_layers - 1) { e2.out = x_out; e2.ldo = D; }
    PROF(DP_PROF_FFN2_GEMM, Path<T>::gemm(s->mid, F, w.w2, m.w2_t, S, D, F, EPI_RESID, e2, st));
  }
  if (!bf) PROF(DP_PROF_CONVERT, launch_from_f32<T>(s->xres, (T*)x_out, S * D, st));
}

extern "C" int dp_stage_forward(dp_stage_t* s, const void* x_in, void* x_out, int32_t n_frames, int32_t frame0,
                                float timestep, void* hip_stream) {
  if (!s || !x_in || !x_out) return fail(DP_EINVAL, "dp_stage_forward: null pointer");
  if (n_frames < 1 || n_frames > s->cfg.max_block_frames)
    return fail(DP_EINVAL, "dp_stage_forward: n_frames %d outside [1, %d]", n_frames, s->cfg.max_block_frames);
  if (frame0 < 0 || (int64_t)frame0 + n_frames > s->cfg.max_abs_frames)
    return fail(DP_EINVAL, "dp_stage_forward: frames [%d, %lld) outside [0, %d)", frame0, (long long)frame0 + n_frames, s->cfg.max_abs_frames);
  if (!(timestep == timestep)) return fail(DP_EINVAL, "dp_stage_forward: timestep is NaN");
  if (s->cache_len > 0 && s->cache0 < s->tok * n_frames && s->cache0 + s->cache_len + s->tok * n_frames > s->Lfit)
    return fail(DP_ESTATE, "dp_stage_forward: no room for the block beside the cached range");   // dp_cache_update rules this out
  hipStream_t st = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  s->launch_ok = true;
  if (s->cfg.dtype == DP_BF16) forward_typed<bf16_t>(s, x_in, x_out, n_frames, frame0, timestep, st);
  else forward_typed<float>(s, x_in, x_out, n_frames, frame0, timestep, st);
  const hipError_t err = hipGetLastError();
  if (err != hipSuccess) return fail(DP_EHIP, "dp_stage_forward: %s", hipGetErrorString(err));
  if (!s->launch_ok) return fail(DP_ESTATE, "dp_stage_forward: a projection's per-head epilogue did not fit its shape");
  s->last_frames = n_frames; s->last_S = s->tok * n_frames;
  return DP_OK;
}

// ------------------------------------------------------------------------------------------ cache
// rows [src, src + n) of every layer's key buffer and columns [src, src + n) of its transposed value buffer
// to [dst, dst + n); the ranges must not overlap
template <typename T>
static void move_cache(dp_stage* s, int64_t src, int64_t dst, int64_t n, hipStream_t st) {
  const int h = s->cfg.n_heads, d = s->cfg.head_dim;
  for (LayerMem& m : s->lm) {
    launch_copy2d<T>((const T*)m.kbuf + src * d, s->Lpad * d, (T*)m.kbuf + dst * d, s->Lpad * d, h, n * d, st);
    launch_copy2d<T>((const T*)m.vtbuf + src, s->Lpad, (T*)m.vtbuf + dst, s->Lpad, (int64_t)h * d, n, st);
  }
}

extern "C" int dp_cache_update(dp_stage_t* s, int32_t first_frame, int32_t n_frames, void* hip_stream) {
  if (!s) return fail(DP_EINVAL, "dp_cache_update: null stage");
  if (n_frames == 0) { s->cache_len = 0; return DP_OK; }
  if (s->last_frames == 0) return fail(DP_ESTATE, "dp_cache_update: no block has been processed yet");
  if (n_frames < 0 || n_frames > s->cfg.max_cache_frames)
    return fail(DP_EINVAL, "dp_cache_update: n_frames %d outside [0, %d]", n_frames, s->cfg.max_cache_frames);
  if (first_frame < 0 || (int64_t)first_frame + n_frames > s->last_frames)
    return fail(DP_EINVAL, "dp_cache_update: frames [%d, %lld) outside the last block's %d frames", first_frame,
                (long long)first_frame + n_frames, s->last_frames);
  const int64_t c0 = s->blk0 + s->tok * first_frame, nc = s->tok * n_frames;
  if (c0 >= s->Smax || c0 + nc + s->Smax <= s->Lfit) {
    // the usual case (always, in the paper's geometry): the frames stay where the last forward wrote them and
    // the next block goes directly before or after them; nothing is copied
    s->cache0 = c0; s->cache_len = nc;
    return DP_OK;
  }
  // A maximal block would fit on neither side: copy the range into the free space beside the last block, at the
  // buffer's start if the last block leaves nc positions free there, else at its end.  One of the two always
  // holds (the buffer has Smax + 2 Ncmax positions, the last block at most Smax, the range lies inside it), and a
  // maximal block then fits behind / before the copy.  The last block stays intact, so a further dp_cache_update
  // can still name other frames of it.
  const int64_t dst = s->blk0 >= nc ? 0 : s->Lfit - nc;
  if (dst != 0 && s->blk0 + s->last_S > dst) return fail(DP_ESTATE, "dp_cache_update: no free space for the retained range");
  hipStream_t st = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  const bool prof = s->prof.begin(DP_PROF_CACHE_COPY, st);
  if (s->cfg.dtype == DP_BF16) move_cache<bf16_t>(s, c0, dst, nc, st); else move_cache<float>(s, c0, dst, nc, st);
  if (prof) s->prof.end(DP_PROF_CACHE_COPY, st);
  const hipError_t err = hipGetLastError();
  if (err != hipSuccess) return fail(DP_EHIP, "dp_cache_update: %s", hipGetErrorString(err));
  s->cache0 = dst; s->cache_len = nc;
  return DP_OK;
}

extern "C" size_t dp_stage_kv_bytes(const dp_stage_config* cfg) {
  const char* why = validate(cfg);
  if (why) { fail(DP_EINVAL, "dp_stage_kv_bytes: %s", why); return 0; }
  const int64_t tok = (int64_t)cfg->tok_h * cfg->tok_w, E = cfg->dtype == DP_BF16 ? 2 : 4;
  const int64_t lpad = rup(tok * cfg->max_block_frames + 2 * tok * cfg->max_cache_frames, 64) + 64;
  return (size_t)(2 * lpad * cfg->dim * E);
}

// ------------------------------------------------------------------------------------------ test hook
template <typename T>
static int peek_typed(dp_stage* s, int what, int layer, float* dst, int64_t cap, int64_t* rows, hipStream_t st) {
  const dp_stage_config& c = s->cfg;
  const int64_t D = c.dim; const int h = c.n_heads, d = c.head_dim;
  const LayerMem& m = s->lm[(size_t)layer];
  int64_t n = 0;
  switch (what) {
    case DP_PEEK_K: case DP_PEEK_V: n = s->last_S; break;
    case DP_PEEK_CACHE_K: case DP_PEEK_CACHE_V: n = s->cache_len; break;
    case DP_PEEK_TEXT_K: case DP_PEEK_TEXT_V: n = c.text_len; break;
    case DP_PEEK_MOD: n = 6; break;
    default: n = s->last_S; break;
  }
  *rows = n;
  if (cap < n * D) return fail(DP_ENOMEM, "dp_stage_peek: need %lld floats", (long long)(n * D));
  if (n == 0) return DP_OK;
  switch (what) {
    case DP_PEEK_K: launch_gather_heads<T>((const T*)m.kbuf, s->Lpad * d, s->blk0, n, h, d, dst, st); break;
    case DP_PEEK_V: launch_gather_vt<T>((const T*)m.vtbuf, s->Lpad, s->blk0, n, h, d, dst, st); break;
    case DP_PEEK_CACHE_K: launch_gather_heads<T>((const T*)m.kbuf, s->Lpad * d, s->cache0, n, h, d, dst, st); break;
    case DP_PEEK_CACHE_V: launch_gather_vt<T>((const T*)m.vtbuf, s->Lpad, s->cache0, n, h, d, dst, st); break;
    case DP_PEEK_TEXT_K: launch_gather_heads<T>((const T*)(s->heads_epi ? m.tkq : m.tk), s->Ltpad * d, 0, n, h, d, dst, st); break;
    case DP_PEEK_TEXT_V: launch_gather_vt<T>((const T*)m.tvt, s->Ltpad, 0, n, h, d, dst, st); break;
    case DP_PEEK_Q:
      if (s->heads_epi) {
        const AttnQNorm qn{s->qssq, s->cross_np, s->Smax, 1.f / (float)D, c.eps, Path<T>::q_scale(d)};
        launch_gather_heads_qnorm((const bf16_t*)s->qbuf, s->Spad * d, n, h, d, qn, dst, st);
      } else {
        launch_gather_heads<T>((const T*)s->qbuf, s->Spad * d, 0, n, h, d, dst, st);
      }
      break;
    case DP_PEEK_ATTN:
      if (!s->tap_attn) return fail(DP_ESTATE, "dp_stage_peek: needs debug_taps");
      launch_to_f32<T>((const T*)s->tap_attn, dst, n * D, st); break;
    case DP_PEEK_CROSS_ATTN: launch_to_f32<T>((const T*)s->attn_o, dst, n * D, st); break;
    case DP_PEEK_X_SELF:
      if (!s->tap_xself) return fail(DP_ESTATE, "dp_stage_peek: needs debug_taps");
      launch_to_f32<float>(s->tap_xself, dst, n * D, st); break;
    case DP_PEEK_X_CROSS:
      if (!s->tap_xcross) return fail(DP_ESTATE, "dp_stage_peek: needs debug_taps");
      launch_to_f32<float>(s->tap_xcross, dst, n * D, st); break;
    case DP_PEEK_X_RES: launch_to_f32<float>(s->xres, dst, n * D, st); break;
    case DP_PEEK_MOD: launch_to_f32<float>(s->mod + (int64_t)layer * 6 * D, dst, 6 * D, st); break;
    default: return fail(DP_EINVAL, "dp_stage_peek: unknown item %d", what);
  }
  return DP_OK;
}

extern "C" int dp_stage_peek(dp_stage_t* s, int32_t what, int32_t layer, float* dst, int64_t capacity, int64_t* rows,
                             void* hip_stream) {
  if (!s || !dst || !rows) return fail(DP_EINVAL, "dp_stage_peek: null pointer");
  if (layer < 0 || layer >= s->cfg.n_layers) return fail(DP_EINVAL, "dp_stage_peek: layer %d out of range", layer);
  const bool needs_fwd = !(what == DP_PEEK_TEXT_K || what == DP_PEEK_TEXT_V || what == DP_PEEK_CACHE_K || what == DP_PEEK_CACHE_V);
  if (needs_fwd && s->last_frames == 0) return fail(DP_ESTATE, "dp_stage_peek: no block has been processed yet");
  hipStream_t st = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  const int rc = s->cfg.dtype == DP_BF16 ? peek_typed<bf16_t>(s, what, layer, dst, capacity, rows, st)
                                         : peek_typed<float>(s, what, layer, dst, capacity, rows, st);
  if (rc != DP_OK) return rc;
  const hipError_t err = hipGetLastError();
  if (err != hipSuccess) return fail(DP_EHIP, "dp_stage_peek: %s", hipGetErrorString(err));
  return DP_OK;
}

// ------------------------------------------------------------------------------------------ measurement hook
extern "C" int dp_stage_profile_begin(dp_stage_t* s, uint32_t class_mask) {
  if (!s) return fail(DP_EINVAL, "dp_stage_profile_begin: null stage");
  Profiler& p = s->prof;
  if (class_mask && p.ev.empty()) {
    try { p.ev.resize(2 * 16384); p.cls.reserve(16384); }
    catch (const std::bad_alloc&) { p.ev.clear(); return fail(DP_ENOMEM, "dp_stage_profile_begin: host allocation failed"); }
    for (size_t i = 0; i < p.ev.size(); ++i) {
      if (hipEventCreate(&p.ev[i]) != hipSuccess) {
        for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(p.ev[j]);
        p.ev.clear();
        return fail(DP_EHIP, "dp_stage_profile_begin: hipEventCreate failed");
      }
    }
  }
  p.mask = class_mask; p.used = 0; p.cls.clear();
  return DP_OK;
}

extern "C" int dp_stage_profile_end(dp_stage_t* s, double* ms, int64_t* launches) {
  if (!s || !ms || !launches) return fail(DP_EINVAL, "dp_stage_profile_end: null pointer");
  Profiler& p = s->prof;
  for (int i = 0; i < DP_PROF_COUNT; ++i) { ms[i] = 0.0; launches[i] = 0; }
  p.mask = 0;
  for (size_t i = 0; i < p.cls.size(); ++i) {
    if (hipEventSynchronize(p.ev[2 * i + 1]) != hipSuccess) return fail(DP_EHIP, "dp_stage_profile_end: hipEventSynchronize failed");
    float t = 0.f;
    if (hipEventElapsedTime(&t, p.ev[2 * i], p.ev[2 * i + 1]) != hipSuccess) return fail(DP_EHIP, "dp_stage_profile_end: hipEventElapsedTime failed");
    ms[p.cls[i]] += (double)t; launches[p.cls[i]] += 1;
  }
  p.used = 0; p.cls.clear();
  return DP_OK;
}
