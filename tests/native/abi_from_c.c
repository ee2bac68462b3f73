/* The header is plain C: this file is compiled as C99 with -pedantic -Werror and linked against
 * libdmm.so.  It plans a small product (host only, no GPU call) and prints what the accessors say. */
#include <stdio.h>

#include "dmm.h"

int main(void) {
  const int64_t rows4[5] = {0, 64, 128, 192, 256}, one[2] = {0, 256}, two[3] = {0, 128, 256};
  dmm_matrix_desc A = {256, 256, 4, 1, rows4, one, 4, 1, 1};
  dmm_matrix_desc B = {256, 256, 2, 2, two, two, 2, 2, 1};
  dmm_matrix_desc C = {256, 256, 2, 2, two, two, 2, 2, 1};
  dmm_plan_t *plan = NULL;
  int rc = dmm_plan(&A, &B, &C, 4, 0u, &plan);
  const dmm_task *t;
  if (rc != DMM_OK) {
    printf("dmm_plan failed: %s\n", dmm_strerror(rc));
    return 1;
  }
  t = dmm_plan_tasks(plan);
  printf("tasks %ld groups %ld items %ld merged %ld first %d:[%ld,%ld)x[%ld,%ld)x[%ld,%ld) tile %d version %d\n",
         (long)dmm_plan_num_tasks(plan), (long)dmm_plan_num_groups(plan), (long)dmm_plan_num_items(plan),
         (long)dmm_plan_num_merged_items(plan), (int)t[0].rank, (long)t[0].m0, (long)t[0].m1, (long)t[0].k0,
         (long)t[0].k1, (long)t[0].n0, (long)t[0].n1, (int)dmm_plan_macro_tile(plan), dmm_version());
  rc = dmm_plan(&A, &B, &C, 4, DMM_STATIONARY_A | DMM_STATIONARY_B, &plan);
  printf("both stationary flags: %d\n", rc);
  dmm_plan_destroy(plan);
  return 0;
}
