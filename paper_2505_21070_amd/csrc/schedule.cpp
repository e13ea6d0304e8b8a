// Host-side queue schedule of block-wise denoising and the paper's bubble-ratio closed forms.
#include <climits>
#include <new>
#include <vector>

#include "../../include/dualparal.h"

int dp_set_error(int code, const char* msg);   // defined next to dp_last_error

// Sec. 3.1: block b (video order, 1-based) enters the queue's tail at diffusion step b at level T;
// every step each queued block is processed once and drops one level; a block leaves after its
// level-1 pass, so at step s the queue holds the blocks with 1 <= T - (s - b) <= T.  Sec. 3.2: a
// block reuses the K/V of the block processed just before it in the same step.  Sec. 3.3: the first
// block may be longer.
extern "C" int dp_blockwise_schedule(const dp_sched_config* cfg, dp_sched_entry* out, int64_t capacity,
                                     int64_t* n_written) {
  if (!cfg || !n_written) return dp_set_error(DP_EINVAL, "dp_blockwise_schedule: null pointer");
  if (cfg->T < 1 || cfg->block_num < 1 || cfg->num_b < 1 || cfg->num_c < 0 || cfg->first_block_frames < 0)
    return dp_set_error(DP_EINVAL, "dp_blockwise_schedule: non-positive size");
  // Sec. 3.2 takes a block's num_c/2 context frames from the ADJACENT block; more than a block holds is undefined
  if (cfg->num_c / 2 > cfg->num_b)
    return dp_set_error(DP_EINVAL, "dp_blockwise_schedule: num_c / 2 exceeds num_b (the context would reach beyond the neighbouring block)");
  if (cfg->order != DP_ORDER_REVERSE && cfg->order != DP_ORDER_SEQUENTIAL)
    return dp_set_error(DP_EINVAL, "dp_blockwise_schedule: unknown order");
  if (cfg->input != DP_INPUT_BLOCK && cfg->input != DP_INPUT_EXTENDED && cfg->input != DP_INPUT_NOCACHE)
    return dp_set_error(DP_EINVAL, "dp_blockwise_schedule: unknown input variant");
  // frame indices and step numbers are 32-bit fields of dp_sched_entry
  const int64_t first64 = cfg->first_block_frames > 0 ? cfg->first_block_frames : cfg->num_b;
  if (first64 + (int64_t)(cfg->block_num - 1) * cfg->num_b + cfg->num_c / 2 > INT32_MAX ||
      (int64_t)cfg->T + cfg->block_num - 1 > INT32_MAX)
    return dp_set_error(DP_EINVAL, "dp_blockwise_schedule: frame or step count beyond 2^31 - 1");
  const int64_t total = (int64_t)cfg->T * cfg->block_num;
  *n_written = total;
  if (capacity < total || !out) return dp_set_error(DP_ENOMEM, "dp_blockwise_schedule: capacity too small");
  const int32_t T = cfg->T, B = cfg->block_num, half = cfg->num_c / 2;
  const int32_t first = cfg->first_block_frames > 0 ? cfg->first_block_frames : cfg->num_b;
  auto frames_of = [&](int32_t b) { return b == 1 ? first : cfg->num_b; };
  auto start_of = [&](int32_t b) { return b == 1 ? 0 : first + (b - 2) * cfg->num_b; };
  auto ctx_of = [&](int32_t b) { const int32_t f = frames_of(b); return half < f ? half : f; };  // frames a neighbour sees
  int64_t n = 0;
  for (int32_t step = 1; step <= T + B - 1; ++step) {
    int32_t lo = step - T + 1; if (lo < 1) lo = 1;        // cleanest block still queued (head)
    int32_t hi = step < B ? step : B;                     // newest block (tail)
    const bool rev = cfg->order == DP_ORDER_REVERSE;
    int32_t prev = 0, prev_keep = 0;
    for (int32_t i = 0; i <= hi - lo; ++i) {
      const int32_t b = rev ? hi - i : lo + i;
      dp_sched_entry e;
      e.step = step; e.block = b; e.level = T - (step - b);
      e.timestep = cfg->t_max * (float)e.level / (float)T;
      e.frame0 = start_of(b); e.n_frames = frames_of(b);
      // Sec. 3.2: frames of the queued neighbours fed along with the block
      const int32_t before = b - 1 >= lo ? ctx_of(b - 1) : 0, after = b + 1 <= hi ? ctx_of(b + 1) : 0;
      int32_t lead = 0, trail = 0;
      if (cfg->input == DP_INPUT_EXTENDED) { if (rev) lead = before; else trail = after; }
      else if (cfg->input == DP_INPUT_NOCACHE) { lead = before; trail = after; }
      e.in_frame0 = e.frame0 - lead; e.in_frames = lead + e.n_frames + trail; e.keep_first = lead;
      e.cache_block = 0; e.cache_first = 0; e.cache_frames = 0;
      if (prev != 0 && half > 0 && cfg->input != DP_INPUT_NOCACHE) {
        e.cache_block = prev;
        e.cache_frames = ctx_of(prev);
        // the neighbour's frames that touch block b, counted from the first frame its pass fed
        e.cache_first = prev_keep + (rev ? 0 : frames_of(prev) - e.cache_frames);
      }
      out[n++] = e;
      prev = b; prev_keep = lead;
    }
  }
  return DP_OK;
}

// Eq. 3 (N <= Block_num), Eq. 4 (N > Block_num), Eq. 5 (sequential order), as printed.
extern "C" double dp_bubble_ratio(int32_t N, int32_t T, int32_t block_num, int32_t order) {
  if (N < 1 || T < 1 || block_num < 1) return -1.0;
  double bubble;
  if (order == DP_ORDER_SEQUENTIAL) bubble = (double)N * N - 1.0;
  else if (order != DP_ORDER_REVERSE) return -1.0;
  else if (N <= block_num) bubble = (double)N * N - N - 1.0;
  else bubble = (double)block_num * (N - T) + (double)N * (T - 2) + 1.0;
  const double all = bubble + (double)T * block_num;
  return all > 0.0 ? bubble / all : -1.0;               // N = T = block_num = 1 is outside the printed forms
}

// Sec. 3.4 / appendix: in-order pipeline of N one-slot stages fed by the queue schedule; a block's next pass waits
// for its previous pass to leave the last stage.
extern "C" int dp_pipeline_simulate(int32_t N, int32_t T, int32_t block_num, int32_t order, int64_t* makespan,
                                    int64_t* bubble_per_device) {
  if (!makespan || !bubble_per_device) return dp_set_error(DP_EINVAL, "dp_pipeline_simulate: null pointer");
  if (N < 1 || T < 1 || block_num < 1) return dp_set_error(DP_EINVAL, "dp_pipeline_simulate: non-positive size");
  if (order != DP_ORDER_REVERSE && order != DP_ORDER_SEQUENTIAL)
    return dp_set_error(DP_EINVAL, "dp_pipeline_simulate: unknown order");
  // the count visits every (pass, device) pair once; beyond 2^34 visits it is refused rather than left running
  if ((double)N * (double)T * (double)block_num > 17179869184.0)
    return dp_set_error(DP_EINVAL, "dp_pipeline_simulate: more than 2^34 device slots to count");
  std::vector<int64_t> free_at, done;
  try {
    free_at.assign((size_t)N, 0);
    done.assign((size_t)block_num + 1, 0);
  } catch (const std::bad_alloc&) {
    return dp_set_error(DP_ENOMEM, "dp_pipeline_simulate: out of host memory");
  }
  for (int64_t step = 1; step <= (int64_t)T + block_num - 1; ++step) {
    int32_t lo = (int32_t)(step - T + 1 < 1 ? 1 : step - T + 1);
    const int32_t hi = (int32_t)(step < block_num ? step : block_num);
    for (int32_t i = 0; i <= hi - lo; ++i) {
      const int32_t b = order == DP_ORDER_REVERSE ? hi - i : lo + i;
      int64_t t = done[(size_t)b];
      for (int32_t j = 0; j < N; ++j) {
        const int64_t start = t > free_at[(size_t)j] ? t : free_at[(size_t)j];
        free_at[(size_t)j] = start + 1;
        t = start + 1;
      }
      done[(size_t)b] = t;
    }
  }
  *makespan = free_at[(size_t)N - 1];
  *bubble_per_device = *makespan - (int64_t)T * block_num;
  return DP_OK;
}

// Sec. 3.3: block 1 is the whole pool; a later block is a shuffle of the pool frames that the last
// num_c/2 frames of the block before it did not use (exactly num_b of them).
extern "C" int dp_noise_assign(const dp_noise_config* cfg, const uint32_t* random_words, int64_t n_words,
                               int32_t* pool_index, int64_t capacity, int64_t* n_written) {
  if (!cfg || !n_written) return dp_set_error(DP_EINVAL, "dp_noise_assign: null pointer");
  if (cfg->block_num < 1 || cfg->num_b < 1 || cfg->num_c < 0)
    return dp_set_error(DP_EINVAL, "dp_noise_assign: bad block_num / num_b / num_c");
  if ((int64_t)cfg->num_b + cfg->num_c / 2 > INT32_MAX)
    return dp_set_error(DP_EINVAL, "dp_noise_assign: pool beyond 2^31 - 1 frames");
  // Sec. 3.3 excludes the noises of the previous block's last num_c/2 frames; a block has only num_b
  if (cfg->num_c / 2 > cfg->num_b)
    return dp_set_error(DP_EINVAL, "dp_noise_assign: num_c / 2 exceeds num_b (a block has no num_c / 2 last frames)");
  const int32_t nb = cfg->num_b, half = cfg->num_c / 2, pool = nb + half;
  const int64_t need_words = (int64_t)(cfg->block_num - 1) * (nb - 1);
  if (n_words < need_words || (need_words > 0 && !random_words))
    return dp_set_error(DP_EINVAL, "dp_noise_assign: too few random words");
  const int64_t total = (int64_t)pool + (int64_t)(cfg->block_num - 1) * nb;
  *n_written = total;
  if (capacity < total || !pool_index) return dp_set_error(DP_ENOMEM, "dp_noise_assign: capacity too small");
  for (int32_t p = 0; p < pool; ++p) pool_index[p] = p;
  const int32_t* tail = pool_index + pool - half;       // pool frames of the previous block's last num_c/2 frames
  int32_t* blk = pool_index + pool;
  int64_t w = 0;
  for (int32_t b = 1; b < cfg->block_num; ++b, blk += nb) {
    int32_t n = 0;
    for (int32_t p = 0; p < pool; ++p) {
      bool used = false;
      for (int32_t t = 0; t < half; ++t) used = used || tail[t] == p;
      if (!used) blk[n++] = p;
    }
    for (int32_t i = nb - 1; i >= 1; --i) {
      const int32_t j = (int32_t)(random_words[w++] % (uint32_t)(i + 1));
      const int32_t tmp = blk[i]; blk[i] = blk[j]; blk[j] = tmp;
    }
    tail = blk + nb - half;
  }
  return DP_OK;
}
