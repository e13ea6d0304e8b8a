// The two ends of the denoising model and the scheduler update (Sec. 2: latent x_t in R^{F x H x W x C} ->
// p = F x H' x W' tokens of hidden size h -> prediction in latent shape -> x_{t-1} = S(eps_t, x_t, t)).
// The paper leaves these steps to the base model; this is a Wan-shaped reading:
//   patch embedding : token (f, y, x) = the 1x2x2 patch (f, 2y+dy, 2x+dx, c), ordered (dy, dx, c), times
//                     W_pe [4C, h] plus b_pe
//   output head     : (shift, scale) = m_head[2, h] + e, e the timestep embedding (before the 6h projection);
//                     LayerNorm(x) (1 + scale) + shift, times W_head [h, 4C] plus b_head, scattered to pixels
//   scheduler step  : flow-matching Euler, x += (sigma_next - sigma) v
// Latents and velocities are fp32; tokens are in the stage's storage type.  The GEMMs, LayerNorm and timestep
// MLP are the stage's kernels.
#include <cstdint>
#include <mutex>
#include <new>

#include "../../include/dualparal.h"
#include "kernels.h"

int dp_set_error(int code, const char* msg);   // defined next to dp_last_error

static inline int64_t rup(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

struct dp_ends {
  dp_ends_config cfg{};
  dp_ends_weights w{};
  int64_t tok, Smax, Spad, P;                  // P = 4 * channels values per token
  void *patches, *h, *w_pe_t, *w_head_t;       // storage type
  float *x32, *out32, *tau, *e1, *e, *mhead, *mod;
};

// token s, value r = (dy*2 + dx)*C + c  <->  latent element ((f*H + 2y+dy)*W + 2x+dx)*C + c
__device__ __forceinline__ int64_t patch_elem(int64_t s, int r, int tok, int tw, int C) {
  const int64_t f = s / tok;
  const int rem = (int)(s % tok), y = rem / tw, x = rem % tw;
  const int dy = r / (2 * C), dx = (r / C) & 1, c = r % C;
  const int64_t H = 2 * (tok / tw), W = 2 * tw;
  return ((f * H + 2 * y + dy) * W + 2 * x + dx) * C + c;
}
template <typename T>
__global__ void k_patchify(const float* __restrict__ latent, T* __restrict__ out, int64_t n, int P, int tok,
                           int tw, int C) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) Elem<T>::st(out + i, latent[patch_elem(i / P, (int)(i % P), tok, tw, C)]);
}
__global__ void k_unpatchify(const float* __restrict__ in, float* __restrict__ latent, int64_t n, int P, int tok,
                             int tw, int C) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) latent[patch_elem(i / P, (int)(i % P), tok, tw, C)] = in[i];
}
__global__ void k_euler(float* __restrict__ x, const float* __restrict__ v, int64_t n, float ds) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) x[i] = x[i] + ds * v[i];
}

static const char* validate(const dp_ends_config* c) {
  if (!c) return "null config";
  if (c->dim < 1 || c->tok_h < 1 || c->tok_w < 1 || c->channels < 1 || c->max_frames < 1) return "non-positive size";
  if (c->dtype != DP_F32 && c->dtype != DP_BF16) return "dtype must be DP_F32 or DP_BF16";
  if (c->freq_dim < 2 || (c->freq_dim & 1)) return "freq_dim must be even";
  if (!(c->eps >= 0.f)) return "bad eps";
  if (c->dim % 8 || c->dim > 8192) return "dim must be a multiple of 8 and at most 8192";
  // upper limits far beyond any model, so that no size below can overflow
  if (c->channels > (1 << 16) || c->freq_dim > (1 << 16) || (int64_t)c->tok_h * c->tok_w > (1 << 24) ||
      (int64_t)c->tok_h * c->tok_w * c->max_frames > (1 << 24))
    return "channels / freq_dim beyond 2^16 or more than 2^24 tokens";
  if (c->dtype == DP_BF16 && (c->dim % 64 || (4 * c->channels) % 64)) return "bf16 path needs dim and 4*channels % 64 == 0";
  return nullptr;
}

static size_t carve(dp_ends* s, void* base) {
  const dp_ends_config& c = s->cfg;
  const int64_t E = c.dtype == DP_BF16 ? 2 : 4, D = c.dim;
  s->tok = (int64_t)c.tok_h * c.tok_w;
  s->Smax = s->tok * c.max_frames;
  s->Spad = rup(s->Smax, 256);
  s->P = 4 * (int64_t)c.channels;
  char* b = (char*)base; size_t off = 0;
  auto take = [&](size_t bytes) { off = (size_t)rup((int64_t)off, 256); void* p = b ? b + off : nullptr; off += bytes; return p; };
  s->patches = take(s->Spad * s->P * E);
  s->h = take(s->Spad * D * E);
  s->x32 = (float*)take(s->Spad * D * 4);
  s->out32 = (float*)take(s->Spad * s->P * 4);
  s->w_pe_t = take(rup(D, 256) * s->P * E);
  s->w_head_t = take(rup(s->P, 256) * D * E);
  s->tau = (float*)take(c.freq_dim * 4);
  s->e1 = (float*)take(GEMV_MAX_SLICES * D * 4); s->e = (float*)take(GEMV_MAX_SLICES * D * 4);   // sliced vectors
  s->mhead = (float*)take(2 * D * 4); s->mod = (float*)take(2 * D * 4);
  return (size_t)rup((int64_t)off, 256);
}

extern "C" size_t dp_ends_workspace_bytes(const dp_ends_config* cfg) {
  const char* why = validate(cfg);
  if (why) { dp_set_error(DP_EINVAL, why); return 0; }
  dp_ends tmp; tmp.cfg = *cfg;
  return carve(&tmp, nullptr);
}

extern "C" int dp_ends_init(const dp_ends_config* cfg, const dp_ends_weights* w, void* workspace,
                            size_t workspace_bytes, void* hip_stream, dp_ends_t** out) {
  if (!out) return dp_set_error(DP_EINVAL, "dp_ends_init: out is null");
  *out = nullptr;
  const char* why = validate(cfg);
  if (why) return dp_set_error(DP_EINVAL, why);
  if (!w || !workspace) return dp_set_error(DP_EINVAL, "dp_ends_init: null pointer");
  const void* const* p = (const void* const*)w;
  for (size_t i = 0; i < sizeof(dp_ends_weights) / sizeof(void*); ++i)
    if (!p[i]) return dp_set_error(DP_EINVAL, "dp_ends_init: null weight pointer");
  if (((uintptr_t)workspace) % 256) return dp_set_error(DP_EINVAL, "dp_ends_init: workspace must be 256-byte aligned");
  dp_ends* s = new (std::nothrow) dp_ends();
  if (!s) return dp_set_error(DP_ENOMEM, "dp_ends_init: out of host memory");
  s->cfg = *cfg; s->w = *w;
  if (carve(s, nullptr) > workspace_bytes) { delete s; return dp_set_error(DP_ENOMEM, "dp_ends_init: workspace too small"); }
  carve(s, workspace);
  hipStream_t st = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  const int64_t D = cfg->dim;
  launch_fill_zero(s->patches, (size_t)((char*)s->tau - (char*)s->patches), st);      // padding rows of the GEMM operands
  if (cfg->dtype == DP_BF16) {
    launch_transpose_pad<bf16_t>((const bf16_t*)w->w_pe, s->P, D, (bf16_t*)s->w_pe_t, rup(D, 256), st);
    launch_transpose_pad<bf16_t>((const bf16_t*)w->w_head, D, s->P, (bf16_t*)s->w_head_t, rup(s->P, 256), st);
    launch_to_f32<bf16_t>((const bf16_t*)w->m_head, s->mhead, 2 * D, st);
  } else {
    launch_to_f32<float>((const float*)w->m_head, s->mhead, 2 * D, st);
  }
  const hipError_t err = hipGetLastError();
  if (err != hipSuccess) { delete s; return dp_set_error(DP_EHIP, "dp_ends_init: a launch failed"); }
  *out = s;
  return DP_OK;
}

extern "C" void dp_ends_free(dp_ends_t* ends) { delete ends; }

template <typename T>
static void gemm(dp_ends* s, const void* A, int64_t lda, const void* W, const void* wt, int64_t M, int64_t N, int64_t K,
                 int epi, const EpiArgs& e, hipStream_t st) {
  if constexpr (sizeof(T) == 2) launch_gemm_bf16((const bf16_t*)A, lda, (const bf16_t*)wt, K, M, N, K, epi, e, st);
  else launch_gemm_f32((const float*)A, lda, (const float*)W, N, M, N, K, epi, e, st);
  (void)s;
}

template <typename T>
static void embed_typed(dp_ends* s, const float* latent, void* x_out, int n_frames, hipStream_t st) {
  const dp_ends_config& c = s->cfg;
  const int64_t S = s->tok * n_frames, n = S * s->P;
  k_patchify<T><<<(unsigned)((n + 255) / 256), 256, 0, st>>>(latent, (T*)s->patches, n, (int)s->P, (int)s->tok, c.tok_w, c.channels);
  gemm<T>(s, s->patches, s->P, s->w.w_pe, s->w_pe_t, S, c.dim, s->P, EPI_STORE, EpiArgs{x_out, c.dim, s->w.b_pe, nullptr, 0, nullptr}, st);
}

extern "C" int dp_embed_forward(dp_ends_t* s, const float* latent, void* x_out, int32_t n_frames, void* hip_stream) {
  if (!s || !latent || !x_out) return dp_set_error(DP_EINVAL, "dp_embed_forward: null pointer");
  if (n_frames < 1 || n_frames > s->cfg.max_frames) return dp_set_error(DP_EINVAL, "dp_embed_forward: n_frames outside [1, max_frames]");
  hipStream_t st = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  if (s->cfg.dtype == DP_BF16) embed_typed<bf16_t>(s, latent, x_out, n_frames, st);
  else embed_typed<float>(s, latent, x_out, n_frames, st);
  if (hipGetLastError() != hipSuccess) return dp_set_error(DP_EHIP, "dp_embed_forward: a launch failed");
  return DP_OK;
}

template <typename T>
static void head_typed(dp_ends* s, const void* x_in, float t, float* v_out, int n_frames, hipStream_t st) {
  const dp_ends_config& c = s->cfg;
  const int64_t D = c.dim, S = s->tok * n_frames, n = S * s->P;
  launch_sinusoid(t, c.freq_dim, s->tau, st);
  launch_gemv<T>(s->tau, 1, 0, (const T*)nullptr, c.freq_dim, (const T*)s->w.wt1, (int)D, 0, s->e1, st);
  launch_gemv<T>(s->e1, gemv_slices(c.freq_dim, (int)D), (int)D, (const T*)s->w.bt1, (int)D, (const T*)s->w.wt2, (int)D, 1, s->e, st);
  launch_mod_add<T>(s->mhead, s->e, gemv_slices((int)D, (int)D), (const T*)s->w.bt2, s->mod, 2, (int)D, st);   // rows: shift, scale
  launch_to_f32<T>((const T*)x_in, s->x32, S * D, st);
  launch_ln_modulate<T>(s->x32, nullptr, (T*)s->h, S, (int)D, c.eps, s->mod + D, s->mod, 1, st);
  // fp32 output through the residual epilogue (out32 += h W + b) on a cleared buffer
  launch_fill_zero(s->out32, (size_t)n * 4, st);
  gemm<T>(s, s->h, D, s->w.w_head, s->w_head_t, S, s->P, D, EPI_RESID, EpiArgs{nullptr, 0, s->w.b_head, s->out32, s->P, nullptr}, st);
  k_unpatchify<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(s->out32, v_out, n, (int)s->P, (int)s->tok, c.tok_w, c.channels);
}

extern "C" int dp_head_forward(dp_ends_t* s, const void* x_in, float timestep, float* v_out, int32_t n_frames,
                               void* hip_stream) {
  if (!s || !x_in || !v_out) return dp_set_error(DP_EINVAL, "dp_head_forward: null pointer");
  if (n_frames < 1 || n_frames > s->cfg.max_frames) return dp_set_error(DP_EINVAL, "dp_head_forward: n_frames outside [1, max_frames]");
  if (!(timestep == timestep)) return dp_set_error(DP_EINVAL, "dp_head_forward: timestep is NaN");
  hipStream_t st = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  if (s->cfg.dtype == DP_BF16) head_typed<bf16_t>(s, x_in, timestep, v_out, n_frames, st);
  else head_typed<float>(s, x_in, timestep, v_out, n_frames, st);
  if (hipGetLastError() != hipSuccess) return dp_set_error(DP_EHIP, "dp_head_forward: a launch failed");
  return DP_OK;
}

// ------------------------------------------------------------------------------------------ no allocation
// dp_head_forward for callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
// that forbid it): no handle and no workspace.  Everything dp_head_forward keeps in the caller's workspace (the
// timestep-MLP vectors, the fp32 copy of the tokens, the normalised tokens, the fp32 result before the scatter,
// the repacked head matrix) lives in one file-scope device array instead.  Each GPU the library runs on holds its
// own copy of the array at its own address, looked up once per device; host code only ever uses that address.
constexpr size_t kHeadScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kHeadScratchBytes];
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[64] = {};                 // by device ordinal; filled on a device's first call

static int head_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
    return dp_set_error(DP_EHIP, "dp_head_forward_static: no current device (or an ordinal beyond 63)");
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p)
      return dp_set_error(DP_EHIP, "dp_head_forward_static: hipGetSymbolAddress failed");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return DP_OK;
}

// the head's share of carve(), sized for the frames of this call
static size_t carve_head(dp_ends* s, void* base, int n_frames) {
  const dp_ends_config& c = s->cfg;
  const int64_t E = c.dtype == DP_BF16 ? 2 : 4, D = c.dim;
  s->tok = (int64_t)c.tok_h * c.tok_w;
  s->Smax = s->tok * n_frames;
  s->Spad = rup(s->Smax, 256);
  s->P = 4 * (int64_t)c.channels;
  char* b = (char*)base; size_t off = 0;
  auto take = [&](size_t bytes) { off = (size_t)rup((int64_t)off, 256); void* p = b ? b + off : nullptr; off += bytes; return p; };
  s->patches = nullptr; s->w_pe_t = nullptr;
  s->h = take(s->Spad * D * E);
  s->x32 = (float*)take(s->Spad * D * 4);
  s->out32 = (float*)take(s->Spad * s->P * 4);
  s->w_head_t = take(rup(s->P, 256) * D * E);
  s->tau = (float*)take(c.freq_dim * 4);
  s->e1 = (float*)take(GEMV_MAX_SLICES * D * 4); s->e = (float*)take(GEMV_MAX_SLICES * D * 4);
  s->mhead = (float*)take(2 * D * 4); s->mod = (float*)take(2 * D * 4);
  return (size_t)rup((int64_t)off, 256);
}

extern "C" int dp_head_forward_static(const dp_ends_config* cfg, const dp_ends_weights* w, const void* x_in,
                                      float timestep, float* v_out, int32_t n_frames, void* hip_stream) {
  const char* why = validate(cfg);
  if (why) return dp_set_error(DP_EINVAL, why);
  if (!w || !x_in || !v_out) return dp_set_error(DP_EINVAL, "dp_head_forward_static: null pointer");
  if (!w->m_head || !w->w_head || !w->b_head || !w->wt1 || !w->bt1 || !w->wt2 || !w->bt2)
    return dp_set_error(DP_EINVAL, "dp_head_forward_static: null weight pointer");
  if (n_frames < 1 || n_frames > cfg->max_frames) return dp_set_error(DP_EINVAL, "dp_head_forward_static: n_frames outside [1, max_frames]");
  if (!(timestep == timestep)) return dp_set_error(DP_EINVAL, "dp_head_forward_static: timestep is NaN");
  dp_ends s;                                            // host struct on the stack: nothing is allocated
  s.cfg = *cfg; s.w = *w;
  if (carve_head(&s, nullptr, n_frames) > kHeadScratchBytes)
    return dp_set_error(DP_ENOMEM, "dp_head_forward_static: this many tokens need more than the 64 MiB of static scratch; "
                                   "call it per frame or use dp_head_forward with a workspace");
  void* base = nullptr;
  const int rc = head_scratch(&base);
  if (rc != DP_OK) return rc;
  carve_head(&s, base, n_frames);
  hipStream_t st = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  const int64_t D = cfg->dim, S = s.tok * n_frames;
  const bool bf = cfg->dtype == DP_BF16;
  // the array keeps the last call's contents: rows of the GEMM operand beyond this call's tokens are cleared with
  // a fill kernel (no memset call, so the entry point can be captured), the rest is overwritten below
  if (s.Spad > S) launch_fill_zero((char*)s.h + S * D * (bf ? 2 : 4), (size_t)((s.Spad - S) * D * (bf ? 2 : 4)), st);
  if (bf) {
    launch_transpose_pad<bf16_t>((const bf16_t*)w->w_head, D, s.P, (bf16_t*)s.w_head_t, rup(s.P, 256), st);
    launch_to_f32<bf16_t>((const bf16_t*)w->m_head, s.mhead, 2 * D, st);
    head_typed<bf16_t>(&s, x_in, timestep, v_out, n_frames, st);
  } else {
    launch_to_f32<float>((const float*)w->m_head, s.mhead, 2 * D, st);
    head_typed<float>(&s, x_in, timestep, v_out, n_frames, st);
  }
  if (hipGetLastError() != hipSuccess) return dp_set_error(DP_EHIP, "dp_head_forward_static: a launch failed");
  return DP_OK;
}

extern "C" int dp_euler_step(float* x, const float* v, int64_t n, float sigma, float sigma_next, void* hip_stream) {
  if (n < 0) return dp_set_error(DP_EINVAL, "dp_euler_step: negative size");
  if (n == 0) return DP_OK;
  if (!x || !v) return dp_set_error(DP_EINVAL, "dp_euler_step: null pointer");
  if (!(sigma == sigma) || !(sigma_next == sigma_next)) return dp_set_error(DP_EINVAL, "dp_euler_step: sigma is NaN");
  (void)hipGetLastError();
  const int64_t blocks = (n + 255) / 256;                      // grid-stride beyond 2^20 blocks: any n fits
  k_euler<<<(unsigned)(blocks < (1 << 20) ? blocks : (1 << 20)), 256, 0, (hipStream_t)hip_stream>>>(x, v, n, sigma_next - sigma);
  if (hipGetLastError() != hipSuccess) return dp_set_error(DP_EHIP, "dp_euler_step: the launch failed");
  return DP_OK;
}
