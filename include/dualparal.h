/*
 * libdualparal -- one GPU's share of DualParal's block-wise denoising, for AMD MI355X (gfx950).
 *
 * A "stage" is the model chunk E_theta_j that one device of the paper's device pipeline owns
 * (Sec. 2, Eq. 1; Sec. 3.1): it receives the hidden tokens eps^{j-1} in R^{p x h} of one frame
 * block, runs them through its consecutive DiT layers and emits eps^j (Sec. 3.2, Eq. 2).  Every
 * layer keeps the self-attention key/value features of the block it processed last (the feature
 * cache of Sec. 3.2); the next block attends over [cached K/V ; its own K/V].  A queue driver
 * (Sec. 3.1) decides which block runs when and at which noise level.
 *
 * Conventions for every entry point
 *  - C linkage, no exceptions; every call returns a DP_* status; dp_last_error() returns a
 *    thread-local text for the last failure on the calling thread.
 *  - "device" pointers are HIP device memory owned by the caller (e.g. torch tensors); "host"
 *    pointers are ordinary host memory, borrowed only for the duration of the call.
 *  - The library never allocates or frees device memory.  All device state of a stage lives in
 *    the caller's workspace, which must outlive the handle.
 *  - Calls that take a stream are asynchronous on it and ordered by it.  One handle is used on
 *    one stream at a time.  `hip_stream` is a hipStream_t passed as void* (NULL = default stream).
 *  - Element type of activations and weights is the config's dtype: DP_F32 (float) or DP_BF16
 *    (bfloat16, upper half of an IEEE float).  Matrices are row-major [in, out]; a stage can also take
 *    them [out, in] (dp_stage_config.weight_layout, see dp_layer_weights).
 */
#ifndef DUALPARAL_H
#define DUALPARAL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dp_stage dp_stage_t; /* opaque, host memory, owned by the library */

enum { DP_OK = 0, DP_EINVAL = -1, DP_ENOMEM = -2 /* workspace / output too small */,
       DP_ESTATE = -3 /* call out of order */, DP_EHIP = -4 /* a HIP call failed */ };
enum { DP_F32 = 0, DP_BF16 = 1 };
/* How the caller hands the weight matrices over (dp_layer_weights, dp_stage_weights). */
enum { DP_WEIGHTS_IN_OUT = 0 /* row-major [in, out]; the bf16 path keeps its own [out, in] copies in the workspace */,
       DP_WEIGHTS_OUT_IN = 1 /* row-major [out, in], as the bf16 GEMMs read them: used in place, no second copy   */ };

/* Geometry of a stage.  All sizes in elements. */
typedef struct {
  int32_t n_layers;           /* consecutive DiT layers this stage owns (L/N of Sec. 2)            */
  int32_t dim;                /* hidden size h                                                    */
  int32_t n_heads, head_dim;  /* n_heads * head_dim == dim; head_dim is 64 or 128                 */
  int32_t ffn_dim;
  int32_t text_len, text_dim; /* text tokens; text_dim != dim adds a two-layer text MLP           */
  int32_t tok_h, tok_w;       /* tokens per latent frame = tok_h * tok_w (H' x W' of Sec. 2)      */
  int32_t max_block_frames;   /* largest block a forward may be given (Num_B [+ Num_C/2])         */
  int32_t max_cache_frames;   /* largest number of cached frames (Num_C/2)                        */
  int32_t max_abs_frames;     /* frame0 + n_frames never exceeds this (extent of the RoPE table)  */
  int32_t dtype;              /* DP_F32 or DP_BF16                                                */
  int32_t freq_dim;           /* width of the sinusoidal timestep features (even)                 */
  float rope_theta;           /* rotary base, e.g. 1e4                                            */
  float eps;                  /* LayerNorm / RMSNorm epsilon, e.g. 1e-6                           */
  int32_t debug_taps;         /* nonzero: keep intermediate results of the last layer for dp_stage_peek */
  int32_t weight_layout;      /* DP_WEIGHTS_IN_OUT or DP_WEIGHTS_OUT_IN (DP_BF16 with dim, ffn_dim % 256 == 0) */
} dp_stage_config;

/* Device pointers to one layer's weights (element type = dtype).  Shapes below are those of DP_WEIGHTS_IN_OUT.
 * With DP_WEIGHTS_OUT_IN every matrix of this struct is its transpose, row-major [out, in], 16-byte aligned:
 * wo, cwq, cwk, cwv, cwo [dim, dim], w1 [ffn_dim, dim], w2 [dim, ffn_dim], and wq, wk, wv are the three row
 * groups of ONE [3 * dim, dim] matrix (wk == wq + dim * dim elements, wv == wq + 2 * dim * dim; anything else is
 * DP_EINVAL).  The stage then multiplies by the caller's memory directly, which halves the weight bytes a device
 * holds (the memory analysis of Sec. 3.1 / Table 1 counts the model chunk once).  Vectors are the same in both. */
typedef struct {
  const void* mod;                               /* [6, dim] rows: shift1, scale1, gate1, shift2, scale2, gate2 */
  const void *wq, *bq, *wk, *bk, *wv, *bv;       /* self-attention projections [dim, dim] / [dim]  */
  const void *gq, *gk;                           /* q / k RMSNorm gains over the full dim          */
  const void *wo, *bo;
  const void *ln3_g, *ln3_b;                     /* affine LayerNorm in front of cross-attention   */
  const void *cwq, *cbq, *cgq, *cwk, *cbk, *cgk, *cwv, *cbv, *cwo, *cbo;
  const void *w1, *b1, *w2, *b2;                 /* FFN [dim, ffn_dim], [ffn_dim], [ffn_dim, dim], [dim] */
} dp_layer_weights;

/* Device pointers to the stage-level weights plus a HOST array of per-layer structs.  With DP_WEIGHTS_OUT_IN
 * the text MLP's wx1 is [dim, text_dim] and wx2 [dim, dim] ([out, in]); wt1, wt2 and wm feed matrix-vector
 * products and stay [in, out] in both layouts. */
typedef struct {
  const void *wt1, *bt1;       /* [freq_dim, dim], [dim]   timestep MLP, first layer               */
  const void *wt2, *bt2;       /* [dim, dim], [dim]                                                */
  const void *wm, *bm;         /* [dim, 6*dim], [6*dim]    modulation head                         */
  const void *wx1, *bx1;       /* [text_dim, dim], [dim]   text MLP (ignored when text_dim == dim) */
  const void *wx2, *bx2;       /* [dim, dim], [dim]                                                */
  const dp_layer_weights* layers; /* host array of n_layers entries                               */
} dp_stage_weights;

/* Bytes of device workspace a stage of this geometry needs (0 if the config is invalid; dp_last_error says
 * why).  Limits besides those stated at the fields: dim <= 8192, n_layers <= 1024, ffn_dim <= 2^17,
 * text_dim <= 2^16, text_len <= 2^20, freq_dim <= 2^16, max_abs_frames <= 2^24, and at most 2^24 tokens
 * (tok_h * tok_w * frames) in a block and in the cache. */
size_t dp_stage_workspace_bytes(const dp_stage_config* cfg);

/*
 * Create a stage (Sec. 2: device j holds the chunk E_theta_j).  Lays the workspace out, repacks the
 * weights it wants in another layout, builds the RoPE tables and runs the text side once per prompt:
 * the optional text MLP and every layer's cross-attention keys/values.  The feature cache starts empty.
 *   cfg, weights : host structs (borrowed); the device memory the weights point to must stay valid
 *                  and unchanged for the life of the handle.
 *   text         : device [text_len, text_dim].
 *   workspace    : device, 256-byte aligned, at least dp_stage_workspace_bytes(cfg) bytes; owned by
 *                  the caller, used exclusively by this handle until dp_stage_free.
 * Errors: DP_EINVAL (null pointer, n_heads*head_dim != dim, unsupported head_dim, sizes the kernels
 * cannot tile), DP_ENOMEM (workspace too small), DP_EHIP.
 */
int dp_stage_init(const dp_stage_config* cfg, const dp_stage_weights* weights, const void* text,
                  void* workspace, size_t workspace_bytes, void* hip_stream, dp_stage_t** out);

/*
 * eps^j = E_theta_j(eps^{j-1}) for one frame block (Sec. 2 Eq. 1, Sec. 3.2 Eq. 2).  For each layer:
 * adaLN-modulated LayerNorm, q/k/v projection with q/k RMSNorm and 3D RoPE at the block's absolute
 * frame offset, self-attention of the block's tokens over [cached K/V ; the block's own K/V]
 * (Sec. 3.2), gated output projection, cross-attention to the text tokens, gated modulated FFN.
 * Cross-attention and FFN touch only the block's own tokens (Sec. 3.2).  The block's rotated keys and
 * values stay in the workspace so that dp_cache_update can retain some of their frames.
 *   x_in  : device [n_frames*tok_h*tok_w, dim], tokens frame-major then row-major.
 *   x_out : device, same shape; may alias x_in.
 *   n_frames in [1, max_block_frames]; frame0 >= 0 is the absolute index of the block's first frame,
 *   frame0 + n_frames <= max_abs_frames; timestep is the block's noise level on the model's
 *   timestep scale (e.g. 0..1000).
 * Asynchronous on hip_stream.  The call allocates nothing, waits for nothing and issues only kernel
 * launches, so it may be recorded into a HIP graph (after one ordinary call, which sets the kernels'
 * attributes); a replay repeats the launch with the pointers, block position and cache range of the
 * moment of capture and does not advance the handle's host-side state.
 * Errors: DP_EINVAL (bad sizes / null), DP_EHIP.
 */
int dp_stage_forward(dp_stage_t* stage, const void* x_in, void* x_out, int32_t n_frames,
                     int32_t frame0, float timestep, void* hip_stream);

/*
 * Feature cache hand-over (Sec. 3.2): in every layer, the cache becomes the rotated keys and the
 * values of frames [first_frame, first_frame + n_frames) of the block the last dp_stage_forward
 * processed (frame indices relative to that block).  The cached keys carry their absolute
 * positions, so the next block may lie before or after them.  n_frames == 0 empties the cache.
 * May be called again for other frames of the same block; the last call counts.
 * In the paper's geometry (blocks of max_block_frames frames handing over their first or last
 * max_cache_frames frames) no data moves and nothing is launched: the frames stay where the forward wrote
 * them, and the next forward writes its own keys and values directly before or after them in the per-layer
 * buffer of max_block_frames + 2 * max_cache_frames frame positions.  Only where a block of max_block_frames
 * frames would fit on neither side of the retained range is the range copied, by kernels on hip_stream (the
 * stream of the forward calls), into the buffer's free space: 2 * n_frames * tok_h * tok_w * dim elements read
 * and written per layer.
 * Errors: DP_ESTATE (no forward yet), DP_EINVAL (range outside the last block or above
 * max_cache_frames), DP_EHIP.
 */
int dp_cache_update(dp_stage_t* stage, int32_t first_frame, int32_t n_frames, void* hip_stream);

/* Bytes of self-attention key/value storage a stage of this geometry keeps per layer (cached range + current
 * block, keys and transposed values): 2 * (max_block_frames + 2 * max_cache_frames) frames of tok_h * tok_w * dim
 * elements, plus at most 127 key positions of alignment padding.  With max_block_frames = Num_B and
 * max_cache_frames = Num_C / 2 that is the (Num_B + Num_C) * KV of the paper's memory analysis (Table 1: KV =
 * one frame's keys and values in one layer).  0 if the config is invalid. */
size_t dp_stage_kv_bytes(const dp_stage_config* cfg);

/* Queue schedule of block-wise denoising (Sec. 3.1, 3.2, 3.3). */
enum { DP_ORDER_REVERSE = 0 /* tail to head, the paper's choice */, DP_ORDER_SEQUENTIAL = 1 /* head to tail */ };
/* What a pass feeds the model (Sec. 3.2).  A neighbour counts only while it is in the queue itself.
 *   DP_INPUT_BLOCK    : the block alone; the neighbour processed just before it is present through the cache
 *   DP_INPUT_EXTENDED : the paper's B_i' = [B_{i-1}, B_i] with the feature cache standing in for B_{i+1}:
 *                       the num_c/2 touching frames of the neighbour processed AFTER this block are fed
 *                       along with it
 *   DP_INPUT_NOCACHE  : B_i' = [B_{i-1}, B_i, B_{i+1}] fed whole, nothing cached (the ablation's baseline) */
enum { DP_INPUT_BLOCK = 0, DP_INPUT_EXTENDED = 1, DP_INPUT_NOCACHE = 2 };

typedef struct {
  int32_t T;                  /* denoising steps = number of noise levels                         */
  int32_t block_num;          /* blocks in the video                                              */
  int32_t num_b;              /* frames per block                                                 */
  int32_t num_c;              /* context frames; a block reuses num_c/2 cached frames of its neighbour */
  int32_t first_block_frames; /* frames of block 1 (Sec. 3.3: num_b + num_c/2); 0 means num_b     */
  int32_t order;              /* DP_ORDER_*                                                       */
  float t_max;                /* timestep of level T; level k maps to t_max * k / T               */
  int32_t input;              /* DP_INPUT_*                                                       */
} dp_sched_config;

typedef struct {
  int32_t step;               /* diffusion step, 1 .. T + block_num - 1                           */
  int32_t block;              /* 1-based block index in video order                               */
  int32_t level;              /* noise level before this pass, T (noisiest) .. 1                  */
  float timestep;
  int32_t frame0, n_frames;   /* absolute first frame and length of the block                     */
  int32_t cache_block;        /* block whose K/V this pass attends to (processed just before); 0 = none */
  int32_t cache_first, cache_frames; /* retained frames of cache_block's pass, relative to the first frame
                                        that pass fed (its in_frame0): the arguments of dp_cache_update   */
  int32_t in_frame0, in_frames; /* the frames to feed dp_stage_forward (= frame0, n_frames for DP_INPUT_BLOCK) */
  int32_t keep_first;         /* offset of the block's own n_frames frames inside the fed frames; the
                                 other output rows are discarded                                     */
} dp_sched_entry;

/*
 * Host only.  Writes the block passes of the whole generation in execution order: block b enters
 * the queue's tail at step b at level T, each step processes every queued block once (tail to head
 * for DP_ORDER_REVERSE), each pass lowers the block's level by one, and a block leaves after its
 * level-1 pass.  There are T * block_num passes.  *n_written receives the number of passes; if
 * capacity is smaller the call writes nothing and returns DP_ENOMEM (out may then be NULL).
 * Errors: DP_EINVAL (null cfg / n_written, non-positive sizes, num_c / 2 > num_b -- Sec. 3.2 takes the context
 * from the adjacent block only --, frame indices or step numbers beyond 2^31 - 1), DP_ENOMEM.
 */
int dp_blockwise_schedule(const dp_sched_config* cfg, dp_sched_entry* out, int64_t capacity,
                          int64_t* n_written);

/* Bubble ratio of the device pipeline as the paper prints it: Eq. 3 / Eq. 4 for DP_ORDER_REVERSE
 * (N <= block_num / N > block_num), Eq. 5 for DP_ORDER_SEQUENTIAL.  Host only.  Returns -1 on bad input
 * (a size below 1, an unknown order, or sizes at which the printed form has no positive denominator). */
double dp_bubble_ratio(int32_t n_devices, int32_t T, int32_t block_num, int32_t order);

/* Slot-level count of the device pipeline that runs the block queue (Sec. 3.1, 3.4, appendix on the denoising
 * order): the model is split over n_devices devices; a block pass occupies devices 1..N for one slot each, in
 * order; a device takes the passes in the queue schedule's order, one at a time; a block's pass of the next
 * diffusion step enters device 1 only after its pass of this step has left device N.  Host only.
 *   makespan          : out, slots until the last pass leaves the last device
 *   bubble_per_device : out, makespan - T * block_num, the idle slots of each device
 * For T > N and block_num >= 2 the count equals the numerators of Eq. 5 and Eq. 4, and (N-1)^2 for the
 * tail-to-head order with N <= block_num (Eq. 3 prints N^2-N-1; dp_bubble_ratio returns the printed forms).
 * Errors: DP_EINVAL (null pointer, non-positive size, unknown order, more than 2^34 (pass, device) slots to
 * count), DP_ENOMEM (host memory). */
int dp_pipeline_simulate(int32_t n_devices, int32_t T, int32_t block_num, int32_t order, int64_t* makespan,
                         int64_t* bubble_per_device);

/*
 * Coordinated noise initialisation (Sec. 3.3, overview figure): every block's initial noise is taken
 * from one shared pool of num_b + num_c/2 frame noises.  Block 1 is the whole pool in its stored order
 * (it is num_c/2 frames longer than the others); each later block is a shuffle of the pool frames that
 * the last num_c/2 frames of the block before it did not use.
 *
 * dp_noise_assign (host only) writes the pool-frame index of every frame of every block, block after
 * block: num_b + num_c/2 entries for block 1, num_b for each later one.  The shuffle is driven by the
 * caller's random words: candidates start in ascending pool index; for position i = num_b-1 .. 1 the
 * entry at i is exchanged with the one at (word mod (i+1)), one word per exchange, consumed in order.
 *   random_words : host, at least (block_num - 1) * (num_b - 1) words (may be NULL if that is 0)
 *   pool_index   : host, out; *n_written receives the number of entries.  capacity too small: nothing
 *                  is written, DP_ENOMEM (pool_index may then be NULL)
 * Errors: DP_EINVAL (null cfg / n_written, block_num < 1, num_b < 1, num_c < 0, num_c / 2 > num_b, too few
 * words, a pool beyond 2^31 - 1 frames), DP_ENOMEM.
 *
 * dp_noise_gather (device) materialises a block's initial noise: out[f, :] = pool[index[f], :].
 *   pool        : device, [pool_frames, frame_bytes] bytes, 16-byte aligned; frame_bytes % 16 == 0
 *   index       : device int32 [n_frames]; entries outside [0, pool_frames) make the kernel write
 *                 zeros for that frame
 *   out         : device, [n_frames, frame_bytes] bytes, 16-byte aligned, must not overlap pool
 * Asynchronous on hip_stream.  n_frames <= 65535; n_frames == 0 is a no-op (pointers are not looked at).  Errors: DP_EINVAL (null pointer, negative size, bad
 * alignment, too many frames).
 */
typedef struct {
  int32_t block_num;          /* blocks in the video                                               */
  int32_t num_b;              /* frames per block (block 1 has num_b + num_c/2)                    */
  int32_t num_c;              /* context frames; the pool holds num_b + num_c/2 frame noises       */
} dp_noise_config;
int dp_noise_assign(const dp_noise_config* cfg, const uint32_t* random_words, int64_t n_words,
                    int32_t* pool_index, int64_t capacity, int64_t* n_written);
int dp_noise_gather(const void* pool, int32_t pool_frames, int64_t frame_bytes, const int32_t* index,
                    int32_t n_frames, void* out, void* hip_stream);

/*
 * The two ends of the model and the scheduler update (Sec. 2: the frame latent x_t in R^{F x H x W x C}
 * becomes p = F x H' x W' tokens of hidden size h, the prediction returns in latent shape, and
 * x_{t-1} = S(eps_t, x_t, t)).  The paper leaves their form to the base model; the reading built here:
 *   patch embedding : token (f, y, x), frame-major then row-major, is the 1x2x2 latent patch
 *                     (f, 2y+dy, 2x+dx, c) flattened with dy slowest and c fastest, times w_pe plus b_pe
 *   output head     : (shift, scale) = m_head[2, dim] + e with e the timestep embedding (sinusoid -> wt1 ->
 *                     SiLU -> wt2, the stage's weights); LayerNorm(x) * (1 + scale) + shift, times w_head
 *                     plus b_head, each token's 4*channels outputs scattered to its patch's pixels
 *   scheduler step  : flow-matching Euler, x <- x + (sigma_next - sigma) * v, sigma = timestep / t_max
 * Latents and velocities are float32 device arrays [n_frames, 2*tok_h, 2*tok_w, channels]; tokens are
 * [n_frames*tok_h*tok_w, dim] in the configured storage type.  Like a stage, the handle owns no device
 * memory: the caller provides the workspace (dp_ends_workspace_bytes, 256-byte aligned) and keeps the
 * weights alive.  Calls are asynchronous on hip_stream.  DP_BF16 needs dim % 64 == 0 and
 * 4 * channels % 64 == 0.
 * Errors: DP_EINVAL (null pointer, sizes outside the configured limits, NaN timestep), DP_ENOMEM
 * (workspace too small), DP_EHIP.
 */
typedef struct dp_ends dp_ends_t;
typedef struct {
  int32_t dim, tok_h, tok_w;  /* as in the stage                                                    */
  int32_t channels;           /* latent channels C; a token carries 4 * C latent values              */
  int32_t max_frames;         /* frames per call                                                     */
  int32_t dtype;              /* DP_F32 or DP_BF16: tokens and weights                               */
  int32_t freq_dim;           /* sinusoidal timestep features, as in the stage                       */
  float eps;                  /* LayerNorm epsilon                                                   */
} dp_ends_config;
typedef struct {              /* device pointers, matrices row-major [in, out], in the storage type  */
  const void *w_pe, *b_pe;    /* [4*channels, dim], [dim]                                            */
  const void *m_head;         /* [2, dim]: shift row, scale row                                      */
  const void *w_head, *b_head;/* [dim, 4*channels], [4*channels]                                     */
  const void *wt1, *bt1, *wt2, *bt2; /* timestep MLP, the same arrays the stages use                 */
} dp_ends_weights;
/* 0 if the config is invalid (dim <= 8192, channels and freq_dim <= 2^16, at most 2^24 tokens). */
size_t dp_ends_workspace_bytes(const dp_ends_config* cfg);
int dp_ends_init(const dp_ends_config* cfg, const dp_ends_weights* weights, void* workspace,
                 size_t workspace_bytes, void* hip_stream, dp_ends_t** out);
int dp_embed_forward(dp_ends_t* ends, const float* latent, void* x_out, int32_t n_frames, void* hip_stream);
int dp_head_forward(dp_ends_t* ends, const void* x_in, float timestep, float* v_out, int32_t n_frames,
                    void* hip_stream);
/* dp_head_forward for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid allocation.  No handle and no workspace: what dp_head_forward keeps in the caller's
 * workspace lives in a 64 MiB device array inside the library (one copy per GPU, held until the process ends),
 * and the call itself allocates nothing, on the device or the host, and issues kernel launches only.
 *   cfg, weights : host structs as for dp_ends_init (w_pe / b_pe are not looked at); cfg->max_frames only bounds
 *                  n_frames
 *   x_in         : device [n_frames*tok_h*tok_w, dim] tokens in cfg->dtype;  v_out : device float32
 *                  [n_frames, 2*tok_h, 2*tok_w, channels], as for dp_head_forward, whose result it reproduces bit
 *                  for bit
 * Size limit: roundup(n_frames*tok_h*tok_w, 256) * (dim * (4 + element size) + 16 * channels) plus a few vectors
 * must fit the 64 MiB (e.g. 4 frames of 30 x 52 tokens at dim 1536 in bf16); beyond it nothing is launched and
 * the call returns DP_ENOMEM.  The output head works token by token, so larger inputs can be fed frame by frame.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two
 * threads) race; calls ordered on one stream do not.  Asynchronous on hip_stream.
 * Errors: DP_EINVAL (null pointer, invalid cfg, n_frames outside [1, max_frames], NaN timestep), DP_ENOMEM (see
 * above), DP_EHIP. */
int dp_head_forward_static(const dp_ends_config* cfg, const dp_ends_weights* weights, const void* x_in,
                           float timestep, float* v_out, int32_t n_frames, void* hip_stream);
/* x[i] += (sigma_next - sigma) * v[i] for n float32 elements; x and v must not overlap. */
int dp_euler_step(float* x, const float* v, int64_t n, float sigma, float sigma_next, void* hip_stream);
void dp_ends_free(dp_ends_t* ends);

/* Test hook: copies an internal result to `dst` as float32, token-major [rows, dim].
 *   what : DP_PEEK_*; layer is used by the K / V / cache / modulation peeks, the others refer to the
 *          last layer the last forward ran (they need cfg.debug_taps for X_SELF / X_CROSS).
 *   dst  : device float buffer of at least `capacity` floats; *rows receives the row count.
 * Errors: DP_ESTATE, DP_EINVAL, DP_ENOMEM. */
enum { DP_PEEK_K = 0, DP_PEEK_V = 1, DP_PEEK_CACHE_K = 2, DP_PEEK_CACHE_V = 3,
       DP_PEEK_Q = 4 /* cross-attention queries of the last layer as the attention kernel uses them; DP_BF16: times
                        log2(e)/sqrt(head_dim), and with dim % 256 == 0 without their RMSNorm gains, which then sit
                        in DP_PEEK_TEXT_K instead */,
       DP_PEEK_ATTN = 5, DP_PEEK_CROSS_ATTN = 6, DP_PEEK_X_SELF = 7, DP_PEEK_X_CROSS = 8,
       DP_PEEK_MOD = 9 /* [6, dim] of `layer` */, DP_PEEK_TEXT_K = 10, DP_PEEK_TEXT_V = 11,
       DP_PEEK_X_RES = 12 /* the fp32 residual stream after the last layer, before rounding to x_out */ };
int dp_stage_peek(dp_stage_t* stage, int32_t what, int32_t layer, float* dst, int64_t capacity,
                  int64_t* rows, void* hip_stream);

/* Measurement hook: per-kernel-class GPU time from HIP events recorded on the caller's stream around
 * the launches of the selected classes.  dp_stage_profile_begin(mask) starts collecting for the classes
 * whose bit (1 << DP_PROF_*) is set (mask 0 stops collecting); dp_stage_profile_end waits for the
 * recorded events and writes, for each of the DP_PROF_COUNT classes, the summed milliseconds and the
 * number of launches into two host arrays, then stops collecting.  At most 16384 launches are recorded
 * per begin/end pair; later ones are not timed.  Events are host-side objects; no device memory is
 * allocated.  DP_PROF_CACHE_COPY reports launches only for the cache hand-overs that had to copy.
 * Errors: DP_EINVAL, DP_EHIP. */
enum { DP_PROF_LN = 0, DP_PROF_QKV_GEMM = 1, DP_PROF_NORM_ROPE = 2, DP_PROF_SELF_ATTN = 3,
       DP_PROF_OPROJ_GEMM = 4, DP_PROF_CROSS_Q_GEMM = 5, DP_PROF_CROSS_ATTN = 6, DP_PROF_CROSS_O_GEMM = 7,
       DP_PROF_FFN1_GEMM = 8, DP_PROF_FFN2_GEMM = 9, DP_PROF_CACHE_COPY = 10, DP_PROF_MODULATION = 11,
       DP_PROF_CONVERT = 12, DP_PROF_COUNT = 13 };
int dp_stage_profile_begin(dp_stage_t* stage, uint32_t class_mask);
int dp_stage_profile_end(dp_stage_t* stage, double* ms /* host [DP_PROF_COUNT] */,
                         int64_t* launches /* host [DP_PROF_COUNT] */);

/* Measurement aid: the rate (TFLOP/s) at which the GPU issues bf16 32x32x16 MFMAs when nothing else
 * happens, 2 wavefronts per SIMD on every compute unit, for all-zero or pseudo-random operand bits.  The
 * clock under matrix load depends on operand bit activity, so the attainable ceiling for real data is
 * below the one for zeros; roofline fractions against the published peak are read next to this figure.
 *   iters         : MFMAs per accumulator (4 accumulators per wavefront); 20000 runs a few milliseconds
 *   scratch       : device buffer of at least 131072 floats that the kernel overwrites
 *   tflops        : host; receives the measured rate
 * Synchronises the stream.  Errors: DP_EINVAL, DP_EHIP. */
enum { DP_PROBE_ZEROS = 0, DP_PROBE_RANDOM = 1 };
int dp_probe_mfma_bf16(int32_t operand_mode, int32_t iters, float* scratch, int64_t scratch_floats,
                       void* hip_stream, double* tflops);

/* Measurement aid: the rate (GB/s, read + written bytes) of a plain streaming pass with the traffic shape of the
 * fused LayerNorm (4 bytes read and 2 bytes written per element): the library's fp32 -> bf16 conversion kernel
 * run `iters` times over n elements, event-timed.  The bandwidth-bound kernels' achieved rates are reported next
 * to this figure, measured in the same run on a buffer of the same size.
 *   src : device float [n];  dst : device bfloat16 [n];  both 16-byte aligned, n a multiple of 8
 * Synchronises the stream.  Errors: DP_EINVAL, DP_EHIP. */
int dp_probe_stream_f32_bf16(const float* src, void* dst, int64_t n, int32_t iters, void* hip_stream,
                             double* gbytes_per_s);

/* Releases the host-side handle (device memory belongs to the caller).  NULL is allowed. */
void dp_stage_free(dp_stage_t* stage);

/* Text of the last error on this thread ("" if none).  The pointer stays valid until the next
 * failing call on the same thread. */
const char* dp_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DUALPARAL_H */
