/* A plain C99 client of the library: the header must compile as C, the symbols must link with C linkage, and
 * the host-only calls must work without a GPU.  Built and run by test_c_client.py. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "dualparal.h"

int main(void) {
  dp_sched_config c;
  memset(&c, 0, sizeof c);
  c.T = 50; c.block_num = 4; c.num_b = 4; c.num_c = 4; c.first_block_frames = 6;
  c.order = DP_ORDER_REVERSE; c.t_max = 1000.0f; c.input = DP_INPUT_BLOCK;
  int64_t n = 0;
  if (dp_blockwise_schedule(&c, NULL, 0, &n) != DP_ENOMEM || n != 200) return 1;
  dp_sched_entry* e = (dp_sched_entry*)malloc((size_t)n * sizeof *e);
  if (!e || dp_blockwise_schedule(&c, e, n, &n) != DP_OK) return 2;
  /* the first pass is block 1 at the noisiest level; the last one is the last block at level 1 */
  if (e[0].block != 1 || e[0].level != 50 || e[n - 1].block != 4 || e[n - 1].level != 1) return 3;
  free(e);
  c.T = 0;
  if (dp_blockwise_schedule(&c, NULL, 0, &n) != DP_EINVAL || strlen(dp_last_error()) == 0) return 4;
  int64_t makespan = 0, bubble = 0;
  if (dp_pipeline_simulate(4, 50, 4, DP_ORDER_REVERSE, &makespan, &bubble) != DP_OK || bubble != 9) return 5;
  if (dp_stage_workspace_bytes(NULL) != 0) return 6;
  printf("ok %.6f\n", dp_bubble_ratio(4, 50, 4, DP_ORDER_REVERSE));
  return 0;
}
