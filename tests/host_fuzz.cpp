// Host-only entry points of the library under AddressSanitizer and UndefinedBehaviorSanitizer: grids of
// small sizes, and extreme sizes that a correct implementation must refuse (or finish) without overflow,
// out-of-bounds access or an exception leaving the C ABI.  Built and run by test_host_sanitized.py together
// with csrc/schedule.cpp; prints "ok <calls>" when nothing tripped.
#include <climits>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "../include/dualparal.h"

int dp_set_error(int code, const char*) { return code; }   // stands in for the library's error string store

static long calls = 0;
#define REQUIRE(c) do { if (!(c)) { std::printf("FAILED %s line %d\n", #c, __LINE__); std::exit(1); } } while (0)

static void schedule_case(int T, int B, int nb, int nc, int first, int order, int input) {
  dp_sched_config c{};
  c.T = T; c.block_num = B; c.num_b = nb; c.num_c = nc; c.first_block_frames = first; c.order = order;
  c.t_max = 1000.f; c.input = input;
  int64_t need = -1;
  int rc = dp_blockwise_schedule(&c, nullptr, 0, &need);
  ++calls;
  if (rc == DP_EINVAL) return;
  REQUIRE(rc == DP_ENOMEM && need == (int64_t)T * B);
  if (need > 200000) return;
  std::vector<dp_sched_entry> out((size_t)need);     // exactly the size asked for: an overrun trips ASan
  int64_t n = 0;
  rc = dp_blockwise_schedule(&c, out.data(), need, &n);
  ++calls;
  REQUIRE(rc == DP_OK && n == need);
  for (const auto& e : out) {
    REQUIRE(e.block >= 1 && e.block <= B && e.level >= 1 && e.level <= T);
    REQUIRE(e.n_frames >= 1 && e.frame0 >= 0 && e.in_frames >= e.n_frames && e.keep_first >= 0);
    REQUIRE(e.in_frame0 >= 0 && e.cache_frames >= 0 && e.cache_first >= 0);
  }
}

static void noise_case(int B, int nb, int nc) {
  dp_noise_config c{B, nb, nc};
  int64_t need = -1;
  const int64_t words = B >= 1 && nb >= 1 ? (int64_t)(B - 1) * (nb - 1) : 0;
  std::vector<uint32_t> w(words > 0 && words < 100000 ? (size_t)words : 0);
  for (size_t i = 0; i < w.size(); ++i) w[i] = (uint32_t)(i * 2654435761u + 12345u);
  int rc = dp_noise_assign(&c, w.empty() ? nullptr : w.data(), (int64_t)w.size(), nullptr, 0, &need);
  ++calls;
  if (rc == DP_EINVAL) return;
  REQUIRE(rc == DP_ENOMEM && need > 0);
  if (need > 200000) return;
  std::vector<int32_t> idx((size_t)need);
  int64_t n = 0;
  rc = dp_noise_assign(&c, w.empty() ? nullptr : w.data(), (int64_t)w.size(), idx.data(), need, &n);
  ++calls;
  REQUIRE(rc == DP_OK && n == need);
  const int pool = nb + nc / 2;
  for (int32_t v : idx) REQUIRE(v >= 0 && v < pool);
}

int main() {
  const int small[] = {1, 2, 3, 4, 5, 7, 8};
  for (int T : small) for (int B : small) for (int nb : {1, 2, 4, 5}) for (int nc : {0, 1, 2, 3, 4, 9})
    for (int first : {0, 1, 6}) for (int order : {0, 1}) for (int input : {0, 1, 2})
      schedule_case(T, B, nb, nc, first, order, input);
  const int wild[] = {INT_MIN, -1, 0, 1, 2, 50, 1 << 16, 1 << 30, INT_MAX - 1, INT_MAX};
  for (int T : wild) for (int B : wild) for (int nb : wild) for (int nc : {-1, 0, 4, INT_MAX})
    for (int first : {-1, 0, INT_MAX}) schedule_case(T, B, nb, nc, first, 0, 1);
  schedule_case(3, 3, 4, 4, 6, 7, 0);
  schedule_case(3, 3, 4, 4, 6, 0, 9);

  for (int B : small) for (int nb : {1, 2, 3, 4, 8}) for (int nc : {0, 1, 2, 4, 6, 16, 17}) noise_case(B, nb, nc);
  for (int B : wild) for (int nb : wild) for (int nc : {-1, 0, 4, INT_MAX - 1, INT_MAX}) noise_case(B, nb, nc);

  for (int N : small) for (int T : small) for (int B : small) for (int order : {0, 1, 2}) {
    int64_t mk = -1, bub = -1;
    const int rc = dp_pipeline_simulate(N, T, B, order, &mk, &bub);
    ++calls;
    if (order == 2) { REQUIRE(rc == DP_EINVAL); continue; }
    REQUIRE(rc == DP_OK && mk >= (int64_t)T * B && bub == mk - (int64_t)T * B);
    const double r = dp_bubble_ratio(N, T, B, order);
    REQUIRE(r >= -1.0 && r < 1.0);                       // the printed forms, finite; -1 = outside their domain
  }
  for (int N : wild) for (int T : wild) for (int B : wild) {
    // only sizes that must be refused: one below 1, or more than 2^34 (pass, device) slots
    if (N > 0 && T > 0 && B > 0 && (double)N * T * B <= 17179869184.0) continue;
    int64_t mk = -1, bub = -1;
    const int rc = dp_pipeline_simulate(N, T, B, 0, &mk, &bub);
    ++calls;
    REQUIRE(rc == DP_EINVAL);
    (void)dp_bubble_ratio(N, T, B, 0); (void)dp_bubble_ratio(N, T, B, 1); (void)dp_bubble_ratio(N, T, B, 5);
  }
  int64_t a, b;
  REQUIRE(dp_pipeline_simulate(1, 1 << 20, 3, 0, &a, &b) == DP_OK && a == 3LL * (1 << 20) && b == 0);
  REQUIRE(dp_pipeline_simulate(4, 50, 4, 0, nullptr, &b) == DP_EINVAL);
  REQUIRE(dp_pipeline_simulate(4, 50, 4, 0, &a, nullptr) == DP_EINVAL);
  REQUIRE(dp_blockwise_schedule(nullptr, nullptr, 0, &a) == DP_EINVAL);
  REQUIRE(dp_noise_assign(nullptr, nullptr, 0, nullptr, 0, &a) == DP_EINVAL);
  std::printf("ok %ld\n", calls);
  return 0;
}
