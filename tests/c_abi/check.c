/* The boundary as a C program sees it: include/raggedshard.h compiled as C99, the host half of the
 * library (plan, queries, CheckValidShard, state-block numbering, error codes) called without a
 * GPU.  Prints "ok" and exits 0, or names the first failed check. */
#include <stdio.h>
#include <string.h>

#include "raggedshard.h"

#define CHECK(cond)                                                 \
  do {                                                              \
    if (!(cond)) {                                                  \
      printf("failed at line %d: %s\n", __LINE__, #cond);           \
      return 1;                                                     \
    }                                                               \
  } while (0)

int main(void) {
  /* the toy unit: six bf16 parameters, four ranks, 16-byte alignment with an FP8 buffer */
  rs_tensor_desc d[6];
  const int64_t rows[6] = {256, 384, 512, 1000, 128, 257};
  const int64_t cols[6] = {384, 0, 256, 128, 128, 130};
  rs_plan* plan = NULL;
  int64_t off[6], bases[7], lo, hi;
  int32_t order[6];
  rs_segment seg[8];
  int i, n;

  memset(d, 0, sizeof d);
  for (i = 0; i < 6; ++i) {
    d[i].rows = rows[i];
    d[i].cols = cols[i];
    d[i].block_mode = cols[i] ? RS_BLOCK_128x128 : RS_BLOCK_1x128;
  }
  CHECK(rs_version() >= 100);
  CHECK(strcmp(rs_strerror(RS_OK), "ok") == 0);
  CHECK(rs_plan_create(d, 6, 4, 16, 1, 0, &plan) == RS_OK && plan != NULL);
  CHECK(rs_plan_num_tensors(plan) == 6 && rs_plan_world(plan) == 4);
  CHECK(rs_plan_payload_elems(plan) == 407554);
  CHECK(rs_plan_shard_elems(plan) % 16 == 0);
  CHECK(rs_plan_total_elems(plan) == 4 * rs_plan_shard_elems(plan));
  CHECK(rs_plan_padding_elems(plan) == rs_plan_total_elems(plan) - 407554);
  CHECK(rs_check_valid_shard(d, 6, 4, 16, 1, 0, rs_plan_shard_elems(plan)) == 1);
  CHECK(rs_check_valid_shard(d, 6, 4, 16, 1, 0, 16) == 0);
  CHECK(rs_plan_offsets(plan, off, 6) == RS_OK && off[0] == 0);
  for (i = 1; i < 6; ++i) CHECK(off[i] >= off[i - 1] + rows[i - 1] * (cols[i - 1] ? cols[i - 1] : 1));
  CHECK(rs_plan_order(plan, order, 6) == RS_OK && order[0] == 0 && order[5] == 5);
  CHECK(rs_plan_scale_bases(plan, bases, 7) == RS_OK && bases[6] == rs_plan_num_scales(plan));
  CHECK(rs_plan_scale_range(plan, 0, &lo, &hi) == RS_OK && lo == 0 && hi > 0);
  CHECK(rs_plan_state_range(plan, 3, &lo, &hi) == RS_OK && hi == rs_plan_num_state_blocks(plan));
  n = rs_plan_rank_segments(plan, 1, seg, 8);
  CHECK(n >= 1 && n <= 8 && seg[0].n > 0 && seg[0].dst_off >= 0);
  /* error paths never crash */
  CHECK(rs_plan_offsets(plan, off, 5) == RS_EINVAL);
  CHECK(rs_plan_scale_range(plan, 4, &lo, &hi) == RS_EINVAL);
  CHECK(rs_pack(plan, NULL, NULL, NULL) == RS_ENOTUPLOADED);
  CHECK(rs_reduce_quantize(plan, 0, NULL, 0, NULL, NULL, NULL, NULL) == RS_ENOTUPLOADED);
  CHECK(rs_adam8_step(plan, 0, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL) == RS_ENOTUPLOADED);
  rs_plan_destroy(plan);
  plan = NULL;
  {
    /* placement helpers: roots by load balancing, the rooted buffer, Shard(dim > 0) granularity */
    int32_t roots[6];
    double loads[4];
    const int64_t shape[3] = {8, 64, 48};
    int64_t g = 0;
    CHECK(rs_select_roots(d, 6, 4, roots, loads) == RS_OK);
    CHECK(roots[1] == -1 && roots[2] == 0 && loads[0] > 0);
    roots[1] = 0;
    CHECK(rs_plan_create_rooted(d, 6, 4, 16, 1, 0, roots, &plan) == RS_OK && plan != NULL);
    CHECK(rs_plan_offsets(plan, off, 6) == RS_OK);
    for (i = 0; i < 6; ++i) CHECK(off[i] / rs_plan_shard_elems(plan) == roots[i]);
    rs_plan_destroy(plan);
    plan = NULL;
    roots[2] = 4;
    CHECK(rs_plan_create_rooted(d, 6, 4, 16, 1, 0, roots, &plan) == RS_EINVAL && plan == NULL);
    CHECK(rs_shard_dim_granularity(shape, 3, 1, 128, &g) == RS_OK && g == 64 * 48);
    CHECK(rs_shard_dim_granularity(shape, 3, 0, 128, &g) == RS_EINVAL);
  }
  d[0].block_mode = 99;
  CHECK(rs_plan_create(d, 6, 4, 16, 1, 0, &plan) == RS_EINVAL && plan == NULL);
  rs_plan_destroy(NULL);
  printf("ok\n");
  return 0;
}
