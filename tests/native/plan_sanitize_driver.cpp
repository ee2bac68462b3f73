// Test driver (host only): runs the library's planner, built with AddressSanitizer and
// UndefinedBehaviorSanitizer, over seeded random descriptors in all three data movement modes,
// with and without the iteration offset and the merged work list, and reads every accessor to its end.  Prints one
// checksum line; any sanitizer report makes the process fail.
#include <cstdint>
#include <cstdio>
#include <vector>

#include "dmm.h"
#include "plan_internal.h"

namespace dmm {
void destroy_device_state(DeviceState *) {}   // the device half is not linked into this driver
}

static uint64_t rng_state = 88172645463325252ull;
static uint64_t rnd() {
  rng_state ^= rng_state << 13;
  rng_state ^= rng_state >> 7;
  rng_state ^= rng_state << 17;
  return rng_state;
}
static int64_t below(int64_t n) { return (int64_t)(rnd() % (uint64_t)n); }

struct Desc {
  std::vector<int64_t> rc, cc;
  dmm_matrix_desc d;
};

static void random_cuts(std::vector<int64_t> *cuts, int64_t dim, int n) {
  cuts->assign((size_t)n + 1, 0);
  (*cuts)[(size_t)n] = dim;
  for (int i = 1; i < n; ++i) (*cuts)[(size_t)i] = below(dim + 1);
  for (int i = 1; i < n; ++i)        // insertion sort of the inner cuts (empty tiles allowed)
    for (int j = i; j > 1 && (*cuts)[(size_t)j] < (*cuts)[(size_t)j - 1]; --j) std::swap((*cuts)[(size_t)j], (*cuts)[(size_t)j - 1]);
}

static void make(Desc *D, int64_t rows, int64_t cols, int p) {
  const int gr = 1 + (int)below(5), gc = 1 + (int)below(5);
  random_cuts(&D->rc, rows, gr);
  random_cuts(&D->cc, cols, gc);
  int c;
  do { c = 1 + (int)below(p); } while (p % c);
  const int per = p / c;
  int pr, pc;
  do { pr = 1 + (int)below(gr); pc = 1 + (int)below(gc); } while (pr * pc > per);
  D->d = {rows, cols, gr, gc, D->rc.data(), D->cc.data(), pr, pc, c};
}

int main() {
  const int ps[] = {1, 2, 3, 4, 6, 8, 12, 16};
  uint64_t sum = 0;
  int plans = 0;
  for (int it = 0; it < 400; ++it) {
    const int p = ps[below(8)];
    const int64_t M = below(700), K = below(700), N = below(700);   // zero extents included
    Desc A, B, C;
    make(&A, M, K, p);
    make(&B, K, N, p);
    make(&C, M, N, p);
    for (uint32_t flags : {0u, 1u, 2u, 4u, 5u, 6u, 8u, 12u}) {
      dmm_plan_t *P = nullptr;
      const int rc = dmm_plan(&A.d, &B.d, &C.d, p, flags, &P);
      if (rc != DMM_OK) { std::printf("plan failed: %s\n", dmm_strerror(rc)); return 1; }
      // the merged work list first: with it the plan has not written out its op list yet
      const int64_t nm = dmm_plan_num_merged_items(P);
      const dmm_merged_item *merged = dmm_plan_merged_items(P);
      for (int64_t i = 0; i < nm; ++i) sum += (uint64_t)(merged[i].m0 + merged[i].n_ext + merged[i].row_pieces + merged[i].col_pieces);
      const int64_t n = dmm_plan_num_tasks(P), g = dmm_plan_num_groups(P), ni = dmm_plan_num_items(P);
      const dmm_task *t = dmm_plan_tasks(P);
      const int64_t *order = dmm_plan_order(P), *offs = dmm_plan_group_offsets(P);
      const dmm_work_item *items = dmm_plan_items(P);
      for (int64_t i = 0; i < n; ++i) sum += (uint64_t)(t[order[i]].m1 + t[i].k0 + t[i].n1 + t[i].rank);
      for (int64_t i = 0; i <= g; ++i) sum += (uint64_t)offs[i];
      for (int64_t i = 0; i < ni; ++i) sum += (uint64_t)(items[i].m0 + items[i].n_ext + items[i].group);
      dmm_plan_destroy(P);
      ++plans;
    }
  }
  // rejected inputs must not leak or touch *out
  {
    Desc A, B, C;
    make(&A, 8, 8, 4);
    make(&B, 9, 8, 4);
    make(&C, 8, 8, 4);
    dmm_plan_t *P = (dmm_plan_t *)0x1;
    if (dmm_plan(&A.d, &B.d, &C.d, 4, 0, &P) != DMM_ESHAPE || P != (dmm_plan_t *)0x1) return 2;
    if (dmm_plan(&A.d, &A.d, &A.d, 4, 3, &P) != DMM_EINVAL || P != (dmm_plan_t *)0x1) return 3;
  }
  std::printf("ok plans=%d checksum=%llu\n", plans, (unsigned long long)sum);
  return 0;
}
