// Host side of the library: slicing planner, task grouping, work-item table.
// Integer arithmetic only; no HIP call is made from this file.
//
//  - op generation: Algorithm 1 (Stationary C) over every virtual rank, with the
//    replication rule of Section 4.1 (replica r of a c-fold replicated C works
//    on the k range [floor(rK/c), floor((r+1)K/c)) and every k bound is clipped
//    to it); on request Algorithm 2 (Stationary B) or its mirror image
//    (Stationary A), whose replicas split M and N respectively in the same
//    way.  overlapping_tiles (Table 1) is answered by binary search on the
//    cut arrays instead of a scan, and "the tiles I own" are enumerated directly
//    from the block-cyclic rule (Section 2.1) instead of testing every tile.
//  - grouping: the paper executes ops in list order (Section 4.2); here ops are
//    regrouped by output sub-tile so one workgroup accumulates all K-segments of
//    a C region in ascending k and writes it once, without atomics.
//  - work items: every group is cut into macro-tiles; the launch order deals
//    blocks of 32 neighbouring macro-tiles to the 8 XCDs in turn (workgroup id
//    modulo 8 selects the XCD, each XCD has its own L2).
#include <algorithm>
#include <cstring>
#include <initializer_list>
#include <new>

#include "plan_internal.h"

namespace dmm {
namespace {

struct Interval {
  int64_t lo, hi;
  bool empty() const { return lo >= hi; }
};

inline Interval meet(Interval a, Interval b) { return {std::max(a.lo, b.lo), std::min(a.hi, b.hi)}; }

// Indices [first, last] of the tiles along one axis that can intersect `iv`
// (empty tiles inside the range still have to be skipped by the caller).
inline void tile_range(const std::vector<int64_t> &cuts, Interval iv, int32_t *first, int32_t *last) {
  if (iv.empty()) { *first = 0; *last = -1; return; }
  // first tile whose upper cut lies above iv.lo
  auto up = std::upper_bound(cuts.begin() + 1, cuts.end(), iv.lo);
  // last tile whose lower cut lies below iv.hi
  auto lo = std::lower_bound(cuts.begin(), cuts.end() - 1, iv.hi);
  *first = (int32_t)(up - (cuts.begin() + 1));
  *last = (int32_t)(lo - cuts.begin()) - 1;
}

int check_cuts(const int64_t *cuts, int32_t n, int64_t dim) {
  if (!cuts || n < 1 || dim < 0) return DMM_EINVAL;
  if (cuts[0] != 0 || cuts[n] != dim) return DMM_EINVAL;
  for (int32_t i = 0; i < n; ++i)
    if (cuts[i + 1] < cuts[i]) return DMM_EINVAL;
  return DMM_OK;
}

int load_grid(const dmm_matrix_desc *d, int32_t nranks, Grid *g) {
  if (d->grid_rows < 1 || d->grid_cols < 1) return DMM_EINVAL;
  int rc = check_cuts(d->row_cuts, d->grid_rows, d->rows);
  if (rc) return rc;
  rc = check_cuts(d->col_cuts, d->grid_cols, d->cols);
  if (rc) return rc;
  if (d->proc_rows < 1 || d->proc_cols < 1) return DMM_EINVAL;
  if (d->replication < 1 || nranks % d->replication != 0) return DMM_EREPL;
  if ((int64_t)d->proc_rows * d->proc_cols > nranks / d->replication) return DMM_EREPL;
  g->rows = d->rows;
  g->cols = d->cols;
  g->gr = d->grid_rows;
  g->gc = d->grid_cols;
  g->rc.assign(d->row_cuts, d->row_cuts + d->grid_rows + 1);
  g->cc.assign(d->col_cuts, d->col_cuts + d->grid_cols + 1);
  g->pr = d->proc_rows;
  g->pc = d->proc_cols;
  g->c = d->replication;
  return DMM_OK;
}

// Ops of one virtual rank, appended in Algorithm 1's loop order.
void generate_rank(const dmm_plan_t &P, int32_t rank, std::vector<dmm_task> *out) {
  const Grid &A = P.A, &B = P.B, &C = P.C;
  const int32_t p = P.nranks;
  const int32_t c_per = p / C.c, a_per = p / A.c, b_per = p / B.c;
  const int32_t c_rep = rank / c_per, a_rep = rank / a_per, b_rep = rank / b_per;
  const int32_t local = rank % c_per;
  if (local >= C.pr * C.pc) return;  // this rank holds no tile of C
  const int32_t my_pr = local / C.pc, my_pc = local % C.pc;
  const int64_t K = A.cols;
  const Interval share{(int64_t)c_rep * K / C.c, ((int64_t)c_rep + 1) * K / C.c};

  for (int32_t i = my_pr; i < C.gr; i += C.pr) {
    const Interval c_rows{C.rc[i], C.rc[i + 1]};
    if (c_rows.empty()) continue;
    int32_t a_r0, a_r1, a_c0, a_c1;
    tile_range(A.rc, c_rows, &a_r0, &a_r1);
    tile_range(A.cc, share, &a_c0, &a_c1);
    for (int32_t j = my_pc; j < C.gc; j += C.pc) {
      const Interval c_cols{C.cc[j], C.cc[j + 1]};
      if (c_cols.empty()) continue;
      int32_t b_c0, b_c1;
      tile_range(B.cc, c_cols, &b_c0, &b_c1);
      for (int32_t ai = a_r0; ai <= a_r1; ++ai) {
        const Interval m = meet(c_rows, {A.rc[ai], A.rc[ai + 1]});
        if (m.empty()) continue;
        for (int32_t aj = a_c0; aj <= a_c1; ++aj) {
          const Interval a_k = meet({A.cc[aj], A.cc[aj + 1]}, share);
          if (a_k.empty()) continue;
          int32_t b_r0, b_r1;
          tile_range(B.rc, a_k, &b_r0, &b_r1);
          for (int32_t bi = b_r0; bi <= b_r1; ++bi) {
            const Interval k = meet(a_k, {B.rc[bi], B.rc[bi + 1]});
            if (k.empty()) continue;
            for (int32_t bj = b_c0; bj <= b_c1; ++bj) {
              const Interval n = meet(c_cols, {B.cc[bj], B.cc[bj + 1]});
              if (n.empty()) continue;
              dmm_task t;
              t.rank = rank;
              t.a_rep = a_rep; t.a_ti = ai; t.a_tj = aj;
              t.b_rep = b_rep; t.b_ti = bi; t.b_tj = bj;
              t.c_rep = c_rep; t.c_ti = i;  t.c_tj = j;
              t.m0 = m.lo; t.m1 = m.hi;
              t.k0 = k.lo; t.k1 = k.hi;
              t.n0 = n.lo; t.n1 = n.hi;
              out->push_back(t);
            }
          }
        }
      }
    }
  }
}

// Ops of one virtual rank with its tiles of B in place (Algorithm 2).  Replica r of a
// c-fold replicated B works on the rows [floor(rM/c), floor((r+1)M/c)) of A and C.
void generate_rank_b(const dmm_plan_t &P, int32_t rank, std::vector<dmm_task> *out) {
  const Grid &A = P.A, &B = P.B, &C = P.C;
  const int32_t p = P.nranks;
  const int32_t c_per = p / C.c, a_per = p / A.c, b_per = p / B.c;
  const int32_t c_rep = rank / c_per, a_rep = rank / a_per, b_rep = rank / b_per;
  const int32_t local = rank % b_per;
  if (local >= B.pr * B.pc) return;  // this rank holds no tile of B
  const int32_t my_pr = local / B.pc, my_pc = local % B.pc;
  const int64_t M = A.rows;
  const Interval share{(int64_t)b_rep * M / B.c, ((int64_t)b_rep + 1) * M / B.c};
  int32_t a_r0, a_r1;
  tile_range(A.rc, share, &a_r0, &a_r1);

  for (int32_t kk = my_pr; kk < B.gr; kk += B.pr) {
    const Interval b_rows{B.rc[kk], B.rc[kk + 1]};
    if (b_rows.empty()) continue;
    int32_t a_c0, a_c1;
    tile_range(A.cc, b_rows, &a_c0, &a_c1);
    for (int32_t j = my_pc; j < B.gc; j += B.pc) {
      const Interval b_cols{B.cc[j], B.cc[j + 1]};
      if (b_cols.empty()) continue;
      int32_t c_c0, c_c1;
      tile_range(C.cc, b_cols, &c_c0, &c_c1);
      for (int32_t ai = a_r0; ai <= a_r1; ++ai) {
        const Interval a_m = meet({A.rc[ai], A.rc[ai + 1]}, share);
        if (a_m.empty()) continue;
        int32_t c_r0, c_r1;
        tile_range(C.rc, a_m, &c_r0, &c_r1);
        for (int32_t aj = a_c0; aj <= a_c1; ++aj) {
          const Interval k = meet({A.cc[aj], A.cc[aj + 1]}, b_rows);
          if (k.empty()) continue;
          for (int32_t ci = c_r0; ci <= c_r1; ++ci) {
            const Interval m = meet(a_m, {C.rc[ci], C.rc[ci + 1]});
            if (m.empty()) continue;
            for (int32_t cj = c_c0; cj <= c_c1; ++cj) {
              const Interval n = meet(b_cols, {C.cc[cj], C.cc[cj + 1]});
              if (n.empty()) continue;
              dmm_task t;
              t.rank = rank;
              t.a_rep = a_rep; t.a_ti = ai; t.a_tj = aj;
              t.b_rep = b_rep; t.b_ti = kk; t.b_tj = j;
              t.c_rep = c_rep; t.c_ti = ci; t.c_tj = cj;
              t.m0 = m.lo; t.m1 = m.hi;
              t.k0 = k.lo; t.k1 = k.hi;
              t.n0 = n.lo; t.n1 = n.hi;
              out->push_back(t);
            }
          }
        }
      }
    }
  }
}

// Ops of one virtual rank with its tiles of A in place (the mirror image of Algorithm 2).
// Replica r of a c-fold replicated A works on the columns [floor(rN/c), floor((r+1)N/c)).
void generate_rank_a(const dmm_plan_t &P, int32_t rank, std::vector<dmm_task> *out) {
  const Grid &A = P.A, &B = P.B, &C = P.C;
  const int32_t p = P.nranks;
  const int32_t c_per = p / C.c, a_per = p / A.c, b_per = p / B.c;
  const int32_t c_rep = rank / c_per, a_rep = rank / a_per, b_rep = rank / b_per;
  const int32_t local = rank % a_per;
  if (local >= A.pr * A.pc) return;  // this rank holds no tile of A
  const int32_t my_pr = local / A.pc, my_pc = local % A.pc;
  const int64_t N = B.cols;
  const Interval share{(int64_t)a_rep * N / A.c, ((int64_t)a_rep + 1) * N / A.c};
  int32_t b_c0, b_c1;
  tile_range(B.cc, share, &b_c0, &b_c1);

  for (int32_t i = my_pr; i < A.gr; i += A.pr) {
    const Interval a_rows{A.rc[i], A.rc[i + 1]};
    if (a_rows.empty()) continue;
    int32_t c_r0, c_r1;
    tile_range(C.rc, a_rows, &c_r0, &c_r1);
    for (int32_t l = my_pc; l < A.gc; l += A.pc) {
      const Interval a_cols{A.cc[l], A.cc[l + 1]};
      if (a_cols.empty()) continue;
      int32_t b_r0, b_r1;
      tile_range(B.rc, a_cols, &b_r0, &b_r1);
      for (int32_t bi = b_r0; bi <= b_r1; ++bi) {
        const Interval k = meet(a_cols, {B.rc[bi], B.rc[bi + 1]});
        if (k.empty()) continue;
        for (int32_t bj = b_c0; bj <= b_c1; ++bj) {
          const Interval b_n = meet({B.cc[bj], B.cc[bj + 1]}, share);
          if (b_n.empty()) continue;
          int32_t c_c0, c_c1;
          tile_range(C.cc, b_n, &c_c0, &c_c1);
          for (int32_t ci = c_r0; ci <= c_r1; ++ci) {
            const Interval m = meet(a_rows, {C.rc[ci], C.rc[ci + 1]});
            if (m.empty()) continue;
            for (int32_t cj = c_c0; cj <= c_c1; ++cj) {
              const Interval n = meet(b_n, {C.cc[cj], C.cc[cj + 1]});
              if (n.empty()) continue;
              dmm_task t;
              t.rank = rank;
              t.a_rep = a_rep; t.a_ti = i;  t.a_tj = l;
              t.b_rep = b_rep; t.b_ti = bi; t.b_tj = bj;
              t.c_rep = c_rep; t.c_ti = ci; t.c_tj = cj;
              t.m0 = m.lo; t.m1 = m.hi;
              t.k0 = k.lo; t.k1 = k.hi;
              t.n0 = n.lo; t.n1 = n.hi;
              out->push_back(t);
            }
          }
        }
      }
    }
  }
}

// Iteration offset of Section 4.2 on one rank's ops [first, end): the ops of each stationary
// tile (a contiguous run) are rotated to start (i + j) positions later in their cyclic order,
// i and j being the tile's grid indices, so that the processes of a process row or column do
// not ask for the same remote tile at the same time.
void apply_iteration_offset(std::vector<dmm_task> *tasks, size_t first, uint32_t stationary) {
  auto tile_of = [stationary](const dmm_task &t, int32_t *i, int32_t *j) {
    if (stationary & DMM_STATIONARY_B) { *i = t.b_ti; *j = t.b_tj; }
    else if (stationary & DMM_STATIONARY_A) { *i = t.a_ti; *j = t.a_tj; }
    else { *i = t.c_ti; *j = t.c_tj; }
  };
  size_t pos = first;
  const size_t end = tasks->size();
  while (pos < end) {
    int32_t i, j, i2, j2;
    tile_of((*tasks)[pos], &i, &j);
    size_t stop = pos + 1;
    for (; stop < end; ++stop) {
      tile_of((*tasks)[stop], &i2, &j2);
      if (i2 != i || j2 != j) break;
    }
    const size_t shift = (size_t)(i + j) % (stop - pos);
    std::rotate(tasks->begin() + pos, tasks->begin() + pos + shift, tasks->begin() + stop);
    pos = stop;
  }
}

struct GroupKey {
  int32_t rep, ti, tj;
  int64_t m0, n0;
  bool operator==(const GroupKey &o) const {
    return rep == o.rep && ti == o.ti && tj == o.tj && m0 == o.m0 && n0 == o.n0;
  }
};

inline GroupKey key_of(const dmm_task &t) { return {t.c_rep, t.c_ti, t.c_tj, t.m0, t.n0}; }

// Sorted, duplicate-free union of cut lists.
std::vector<int64_t> merged_cuts(std::initializer_list<const std::vector<int64_t> *> lists) {
  std::vector<int64_t> out;
  for (const std::vector<int64_t> *l : lists) out.insert(out.end(), l->begin(), l->end());
  std::sort(out.begin(), out.end());
  out.erase(std::unique(out.begin(), out.end()), out.end());
  return out;
}

// position of every cut of `cuts` in `merged` (which contains them all)
std::vector<int32_t> ranks_in(const std::vector<int64_t> &merged, const std::vector<int64_t> &cuts) {
  std::vector<int32_t> r(cuts.size());
  for (size_t i = 0; i < cuts.size(); ++i)
    r[i] = (int32_t)(std::lower_bound(merged.begin(), merged.end(), cuts[i]) - merged.begin());
  return r;
}

// The general grouping: a comparison sort on (output sub-tile, k, original position).
void sort_order_by_comparison(dmm_plan_t *P) {
  const auto &T = P->tasks;
  std::sort(P->order.begin(), P->order.end(), [&T](int64_t x, int64_t y) {
    const dmm_task &a = T[x], &b = T[y];
    if (a.c_rep != b.c_rep) return a.c_rep < b.c_rep;
    if (a.c_ti != b.c_ti) return a.c_ti < b.c_ti;
    if (a.c_tj != b.c_tj) return a.c_tj < b.c_tj;
    if (a.m0 != b.m0) return a.m0 < b.m0;
    if (a.n0 != b.n0) return a.n0 < b.n0;
    if (a.k0 != b.k0) return a.k0 < b.k0;
    return x < y;
  });
}

// The same order without comparing tasks: an op's m0 is the largest of a few cut points (the
// lower cuts of its C tile row and A tile row, and of its replica's share of M with Stationary
// B), so its position among the merged row cuts is the largest of their positions, read from
// small tables; likewise n0.  That numbers every possible output sub-tile densely; a table walks
// them in (replica, tile row, tile column, m0, n0) order, a counting sort (stable) puts the ops
// into their groups, and a group whose ops did not arrive in ascending k is sorted on its own.
// Returns false (nothing done) when the dense numbering would be much larger than the op list.
bool sort_order_by_counting(dmm_plan_t *P, uint32_t flags) {
  const auto &T = P->tasks;
  const size_t n = T.size();
  const Grid &A = P->A, &B = P->B, &C = P->C;
  std::vector<int64_t> m_share, n_share;                 // share boundaries of a replicated stationary B / A
  if (flags & DMM_STATIONARY_B)
    for (int32_t r = 0; r <= B.c; ++r) m_share.push_back((int64_t)r * A.rows / B.c);
  if (flags & DMM_STATIONARY_A)
    for (int32_t r = 0; r <= A.c; ++r) n_share.push_back((int64_t)r * B.cols / A.c);
  const std::vector<int64_t> mc = merged_cuts({&A.rc, &C.rc, &m_share}), nc = merged_cuts({&B.cc, &C.cc, &n_share});
  const size_t MR = mc.size(), NR = nc.size();
  const size_t dense = (size_t)C.c * MR * NR;
  if (dense > 4 * n + 4096) return false;
  const std::vector<int32_t> ra = ranks_in(mc, A.rc), rcr = ranks_in(mc, C.rc), rms = ranks_in(mc, m_share);
  const std::vector<int32_t> rb = ranks_in(nc, B.cc), rcc = ranks_in(nc, C.cc), rns = ranks_in(nc, n_share);
  std::vector<uint32_t> gid(n);
  std::vector<int64_t> count(dense + 1, 0);
  for (size_t i = 0; i < n; ++i) {
    const dmm_task &t = T[i];
    int32_t mr = std::max(ra[(size_t)t.a_ti], rcr[(size_t)t.c_ti]);
    int32_t nr = std::max(rb[(size_t)t.b_tj], rcc[(size_t)t.c_tj]);
    if (!rms.empty()) mr = std::max(mr, rms[(size_t)t.b_rep]);
    if (!rns.empty()) nr = std::max(nr, rns[(size_t)t.a_rep]);
    if (mc[(size_t)mr] != t.m0 || nc[(size_t)nr] != t.n0) return false;   // not of the expected form: general sort
    const size_t g = ((size_t)t.c_rep * MR + (size_t)mr) * NR + (size_t)nr;
    gid[i] = (uint32_t)g;
    ++count[g];
  }
  // first position of every dense number, walking them in group order
  std::vector<int64_t> start(dense, 0);
  int64_t run = 0;
  for (int32_t rep = 0; rep < C.c; ++rep)
    for (int32_t ti = 0; ti < C.gr; ++ti)
      for (int32_t tj = 0; tj < C.gc; ++tj)
        for (int32_t mr = rcr[(size_t)ti]; mr < rcr[(size_t)ti + 1]; ++mr)
          for (int32_t nr = rcc[(size_t)tj]; nr < rcc[(size_t)tj + 1]; ++nr) {
            const size_t g = ((size_t)rep * MR + (size_t)mr) * NR + (size_t)nr;
            start[g] = run;
            run += count[g];
          }
  if (run != (int64_t)n) return false;
  for (size_t i = 0; i < n; ++i) P->order[(size_t)start[gid[i]]++] = (int64_t)i;
  // inside a group: ascending k, ties (none in a valid plan) by original position
  size_t pos = 0;
  while (pos < n) {
    const uint32_t g = gid[(size_t)P->order[pos]];
    size_t end = pos + 1;
    bool ascending = true;
    for (; end < n && gid[(size_t)P->order[end]] == g; ++end)
      if (T[(size_t)P->order[end]].k0 < T[(size_t)P->order[end - 1]].k0) ascending = false;
    if (!ascending)
      std::stable_sort(P->order.begin() + pos, P->order.begin() + end,
                       [&T](int64_t x, int64_t y) { return T[(size_t)x].k0 < T[(size_t)y].k0; });
    pos = end;
  }
  return true;
}

void group_tasks(dmm_plan_t *P, uint32_t flags) {
  const auto &T = P->tasks;
  const int64_t n = (int64_t)T.size();
  P->order.resize(n);
  // total order: output sub-tile, then k, then original position (= stable)
  if (n > (int64_t)UINT32_MAX || !sort_order_by_counting(P, flags)) {
    for (int64_t i = 0; i < n; ++i) P->order[i] = i;
    sort_order_by_comparison(P);
  }
  P->group_offsets.clear();
  P->groups.clear();
  for (int64_t pos = 0; pos < n; ++pos) {
    const dmm_task &t = T[P->order[pos]];
    if (pos == 0 || !(key_of(t) == key_of(T[P->order[pos - 1]]))) {
      P->group_offsets.push_back(pos);
      P->groups.push_back({t.m0, t.m1, t.n0, t.n1, t.c_rep, t.c_ti, t.c_tj, pos, 0});
    }
    P->groups.back().count++;
  }
  P->group_offsets.push_back(n);
}

// Macro-tiles of one output region, appended in an order whose every run of 32
// consecutive entries is a compact 4 x 8 block of macro-tiles (the workgroups of
// one XCD that run together then share A row panels and B column panels in L2).
void tile_region(int64_t group, int64_t m0, int64_t m1, int64_t n0, int64_t n1, int32_t rep, int32_t ti,
                 int32_t tj, std::vector<dmm_work_item> *seq) {
  const int64_t T = kMacroTile;
  const int64_t tm = (m1 - m0 + T - 1) / T, tn = (n1 - n0 + T - 1) / T;
  const int64_t strip = 8, band = 4;
  for (int64_t s = 0; s < tn; s += strip)
    for (int64_t r0 = 0; r0 < tm; r0 += band)
      for (int64_t r = r0; r < std::min(tm, r0 + band); ++r)
        for (int64_t c = s; c < std::min(tn, s + strip); ++c) {
          dmm_work_item it;
          it.group = group;
          it.m0 = m0 + r * T;
          it.n0 = n0 + c * T;
          it.m_ext = (int32_t)std::min<int64_t>(T, m1 - it.m0);
          it.n_ext = (int32_t)std::min<int64_t>(T, n1 - it.n0);
          it.c_rep = rep; it.c_ti = ti; it.c_tj = tj;
          it.reserved = 0;
          seq->push_back(it);
        }
}

// Launch slot i goes to XCD i % 8.  Two ways of dealing a sequence of macro-tiles (whose every run
// of 32 is a compact block) to the 8 XCDs:
//  - round-robin in blocks of 32 (the CUs of one XCD): at any time the 8 XCDs work on 8
//    consecutive blocks, i.e. on neighbouring bands of the same column strip of one output
//    region, which read the same B column panels (and the same replica of A) at about the same
//    time, so that what one XCD pulled into the last-level cache serves the other seven;
//  - 8 contiguous runs: each XCD on a region of its own.
// The first wins where strips hold several bands (against the second: cfg3 +6 %, cfg5 +10 %,
// column-block MLP-2 +24 %, cfg4 the same); where every strip is a single band, consecutive
// blocks share no B panel and streaming separate regions is the better of the two (inner-
// product MLP-1: +5 %).
template <typename Item>
void deal_to_xcds(const std::vector<Item> &seq, bool round_robin, std::vector<Item> *out) {
  const int64_t n = (int64_t)seq.size(), X = 8, BLK = 32;
  out->clear();
  out->reserve((size_t)n);
  if (round_robin) {
    const int64_t nblk = (n + BLK - 1) / BLK;
    for (int64_t b0 = 0; b0 < nblk; b0 += X)
      for (int64_t j = 0; j < BLK; ++j)
        for (int64_t x = 0; x < X; ++x) {
          const int64_t idx = (b0 + x) * BLK + j;
          if (idx < n) out->push_back(seq[(size_t)idx]);
        }
  } else {
    int64_t longest = 0;
    for (int64_t x = 0; x < X; ++x) longest = std::max(longest, (x + 1) * n / X - x * n / X);
    for (int64_t j = 0; j < longest; ++j)
      for (int64_t x = 0; x < X; ++x) {
        const int64_t b0 = x * n / X, e = (x + 1) * n / X;
        if (b0 + j < e) out->push_back(seq[(size_t)(b0 + j)]);
      }
  }
}

void build_items(dmm_plan_t *P) {
  std::vector<dmm_work_item> seq;
  for (size_t g = 0; g < P->groups.size(); ++g) {
    const Group &G = P->groups[g];
    tile_region((int64_t)g, G.m0, G.m1, G.n0, G.n1, G.c_rep, G.c_ti, G.c_tj, &seq);
  }
  // Every element of every C replica has to be defined.  Regions no group writes hold a
  // partial sum of zero: a replica of a stationary C whose share of k is empty; with
  // Stationary B or A, the parts of a C replica that none of its ranks' ops update.  Zero-fill
  // items cover, per C tile, the complement of its groups' rectangles (the rectangles are
  // cells of one grid: the cuts of all of them, taken together).
  const Grid &C = P->C;
  size_t g = 0;                                   // groups are sorted by (replica, tile row, tile column)
  std::vector<int64_t> mc, nc;
  std::vector<char> covered;
  for (int32_t rep = 0; rep < C.c; ++rep)
    for (int32_t ti = 0; ti < C.gr; ++ti)
      for (int32_t tj = 0; tj < C.gc; ++tj) {
        const size_t g0 = g;
        while (g < P->groups.size() && P->groups[g].c_rep == rep && P->groups[g].c_ti == ti &&
               P->groups[g].c_tj == tj)
          ++g;
        if (C.rc[ti] >= C.rc[ti + 1] || C.cc[tj] >= C.cc[tj + 1]) continue;
        mc.assign({C.rc[ti], C.rc[ti + 1]});
        nc.assign({C.cc[tj], C.cc[tj + 1]});
        for (size_t q = g0; q < g; ++q) {
          mc.push_back(P->groups[q].m0); mc.push_back(P->groups[q].m1);
          nc.push_back(P->groups[q].n0); nc.push_back(P->groups[q].n1);
        }
        std::sort(mc.begin(), mc.end()); mc.erase(std::unique(mc.begin(), mc.end()), mc.end());
        std::sort(nc.begin(), nc.end()); nc.erase(std::unique(nc.begin(), nc.end()), nc.end());
        const size_t nm = mc.size() - 1, nn = nc.size() - 1;
        covered.assign(nm * nn, 0);
        for (size_t q = g0; q < g; ++q) {
          const Group &G = P->groups[q];
          const size_t i0 = std::lower_bound(mc.begin(), mc.end(), G.m0) - mc.begin();
          const size_t i1 = std::lower_bound(mc.begin(), mc.end(), G.m1) - mc.begin();
          const size_t j0 = std::lower_bound(nc.begin(), nc.end(), G.n0) - nc.begin();
          const size_t j1 = std::lower_bound(nc.begin(), nc.end(), G.n1) - nc.begin();
          for (size_t i = i0; i < i1; ++i)
            for (size_t j = j0; j < j1; ++j) covered[i * nn + j] = 1;
        }
        for (size_t i = 0; i < nm; ++i)
          for (size_t j = 0; j < nn;) {
            if (covered[i * nn + j]) { ++j; continue; }
            size_t e = j;
            while (e < nn && !covered[i * nn + e]) ++e;      // a run of uncovered cells in this row band
            tile_region(-1, mc[i], mc[i + 1], nc[j], nc[e], rep, ti, tj, &seq);
            j = e;
          }
      }
  int64_t blocks = 0, followed = 0;
  for (const Group &G : P->groups) {
    const int64_t T = kMacroTile;
    const int64_t bands = ((G.m1 - G.m0 + T - 1) / T + 3) / 4, strips = ((G.n1 - G.n0 + T - 1) / T + 7) / 8;
    blocks += bands * strips;
    followed += (bands - 1) * strips;
  }
  deal_to_xcds(seq, 2 * followed >= blocks, &P->items);
}

// One axis of a C replica cut into macro-tile extents: 256 at a time, across the cuts; a tile
// ends early where it would meet more than `cap` intervals, or at a cut that is not a multiple
// of `align` away from the tile's start.
struct Extent {
  int64_t start;
  int32_t ext, first, pieces;         // first interval met, number of intervals met
};

std::vector<Extent> tile_axis(const std::vector<int64_t> &cuts, int32_t cap, int64_t align) {
  std::vector<Extent> out;
  const int64_t L = cuts.back();
  int64_t pos = 0;
  size_t iv = 0;
  while (pos < L) {
    while (cuts[iv + 1] <= pos) ++iv;
    int64_t end = std::min<int64_t>(pos + kMacroTile, L);
    int32_t pieces = 1;
    for (size_t j = iv; cuts[j + 1] < end; ++j) {
      const int64_t c = cuts[j + 1];
      if (pieces == cap || (c - pos) % align != 0) {
        end = c;
        break;
      }
      ++pieces;
    }
    out.push_back({pos, (int32_t)(end - pos), (int32_t)iv, pieces});
    pos = end;
  }
  return out;
}

void build_merged(dmm_plan_t *P, uint32_t flags) {
  Merged &G = P->merged;
  G = Merged();
  const Grid &A = P->A, &B = P->B, &C = P->C;
  // With B or A in place the ops are the same boxes as with C in place as long as nothing is
  // replicated (only the rank that performs a box differs), so the same work list serves; their
  // replicas split M or N instead of K, which this list does not describe.
  if ((flags & (DMM_STATIONARY_B | DMM_STATIONARY_A)) && (A.c != 1 || B.c != 1 || C.c != 1)) return;
  const int64_t M = A.rows, K = A.cols, N = B.cols, lim = (int64_t)1 << 31;
  if (M <= 0 || K <= 0 || N <= 0 || M >= lim || K >= lim || N >= lim) return;
  G.mc = merged_cuts({&A.rc, &C.rc});
  G.nc = merged_cuts({&B.cc, &C.cc});
  const std::vector<int64_t> kall = merged_cuts({&A.cc, &B.rc});
  int64_t cap = kMaxPieces, longest = 0;
  for (int32_t rep = 0; rep < C.c; ++rep) {
    const int64_t lo = (int64_t)rep * K / C.c, hi = ((int64_t)rep + 1) * K / C.c;
    if (lo >= hi) return;             // an empty share: that replica is zero-filled, not multiplied
    MergedRep R;
    R.kc.push_back(lo);
    for (int64_t c : kall)
      if (c > lo && c < hi) R.kc.push_back(c);
    R.kc.push_back(hi);
    // One replica of A and one of B serve all macro-tiles of a C replica.  Where the replication
    // factor of A (B) divides that of C this is the replica every rank of the C replica reads by
    // the replication rule (Section 4.1).  Otherwise the ranks of one C replica read several
    // replicas of A (B), tile by tile, which a macro-tile across tiles cannot follow; replicas of
    // an input are copies of each other (Section 3), so reading the first of them gives the same
    // product, bit for bit.  (The op list, written out by materialize, keeps the rule's replica.)
    R.a_rep = (int32_t)((int64_t)rep * A.c / C.c);
    R.b_rep = (int32_t)((int64_t)rep * B.c / C.c);
    const int64_t S = (int64_t)R.kc.size() - 1;
    cap = std::min(cap, (kDescBytes - 4 * ((S + 3) & ~(int64_t)3)) / (48 * S));
    longest = std::max(longest, S);
    G.reps.push_back(std::move(R));
  }
  if (cap < kMinPieces && longest > kSegWindow) {
    // many short segments (K long against the tiles): rather than small macro-tiles, full ones that
    // are run kSegWindow segments at a time
    static_assert(4 * kSegWindow + 48 * kSegWindow * kMaxPieces <= kDescBytes, "a window of segments with all pieces fits");
    G.window = kSegWindow;
    cap = kMaxPieces;
  }
  if (cap < 1) return;
  {
    // the device tables hold one slice per (row interval, segment), (segment, column interval) and
    // (row interval, column interval) of every replica, indexed with 32 bits: keep them moderate
    const double mr = (double)G.mc.size(), nr = (double)G.nc.size();
    double slices = 0;
    for (const MergedRep &R : G.reps) slices += (mr + nr) * (double)R.kc.size() + mr * nr;
    if (slices > 1.6e7) return;
  }
  const std::vector<Extent> rows = tile_axis(G.mc, (int32_t)cap, 1), cols = tile_axis(G.nc, (int32_t)cap, kPieceAlign);
  // worth it only if it saves a tenth of the macro-tiles
  const int64_t merged_count = (int64_t)C.c * (int64_t)rows.size() * (int64_t)cols.size();
  if (!(flags & DMM_MERGE_ALWAYS)) {
    // (macro-tiles of the other list: every cell of the refinement grid tiled on its own)
    int64_t tr = 0, tc = 0;
    for (size_t i = 0; i + 1 < G.mc.size(); ++i) tr += (G.mc[i + 1] - G.mc[i] + kMacroTile - 1) / kMacroTile;
    for (size_t j = 0; j + 1 < G.nc.size(); ++j) tc += (G.nc[j + 1] - G.nc[j] + kMacroTile - 1) / kMacroTile;
    // ... or where the op list is so long against the work list (16 ops and more per macro-tile,
    // thousands in all) that writing it out and turning it into device tables on every call costs
    // the host as long as the multiplication takes the device (8192^3 in 256 x 256 tiles: 32768 ops,
    // 1.4 ms of host time against 0.1 ms for the factored form and 0.95 ms of device time)
    int64_t ops = 0;
    for (const MergedRep &R : G.reps) ops += (int64_t)(G.mc.size() - 1) * (int64_t)(G.nc.size() - 1) * (int64_t)(R.kc.size() - 1);
    const int64_t simple_count = (int64_t)C.c * tr * tc;
    const bool saves_tiles = merged_count * 10 <= simple_count * 9;
    const bool saves_host = ops >= 4096 && ops >= 16 * simple_count;
    if (!saves_tiles && !saves_host) return;
  }
  std::vector<MergedItem> seq;
  seq.reserve((size_t)merged_count);
  const int64_t tm = (int64_t)rows.size(), tn = (int64_t)cols.size(), strip = 8, band = 4;
  for (int32_t rep = 0; rep < C.c; ++rep)
    for (int64_t s = 0; s < tn; s += strip)
      for (int64_t r0 = 0; r0 < tm; r0 += band)
        for (int64_t r = r0; r < std::min(tm, r0 + band); ++r)
          for (int64_t c = s; c < std::min(tn, s + strip); ++c) {
            const Extent &er = rows[(size_t)r], &ec = cols[(size_t)c];
            seq.push_back({er.start, ec.start, er.ext, ec.ext, rep, er.first, er.pieces, ec.first, ec.pieces});
          }
  deal_to_xcds(seq, tm > band, &G.items);
  G.view.reserve(G.items.size());
  for (const MergedItem &w : G.items) G.view.push_back({w.m0, w.n0, w.m_ext, w.n_ext, w.rep, w.R, w.Q, 0});
  G.valid = true;
}

}  // namespace

int materialize(dmm_plan_t *P) {
  if (P->listed) return DMM_OK;
  const uint32_t flags = P->flags;
  try {
    P->tasks.clear();
    {
      // room for the op list up front: the boxes are cells of the merged cut grids (at most one
      // more k interval per replica share), so their number is known to within that
      const size_t mi = merged_cuts({&P->A.rc, &P->C.rc}).size(), ni = merged_cuts({&P->B.cc, &P->C.cc}).size();
      const size_t ki = merged_cuts({&P->A.cc, &P->B.rc}).size() + (size_t)P->C.c;
      const double est = (double)mi * (double)ni * (double)ki;
      if (est < 5.0e7) P->tasks.reserve((size_t)est);
    }
    for (int32_t rank = 0; rank < P->nranks; ++rank) {
      const size_t first = P->tasks.size();
      if (flags & DMM_STATIONARY_B) generate_rank_b(*P, rank, &P->tasks);
      else if (flags & DMM_STATIONARY_A) generate_rank_a(*P, rank, &P->tasks);
      else generate_rank(*P, rank, &P->tasks);
      if (flags & DMM_ITERATION_OFFSET) apply_iteration_offset(&P->tasks, first, flags);
    }
    group_tasks(P, flags);
    build_items(P);
  } catch (const std::bad_alloc &) {
    P->tasks.clear();
    P->order.clear();
    P->group_offsets.clear();
    P->groups.clear();
    P->items.clear();
    return DMM_ENOMEM;
  }
  P->listed = true;
  return DMM_OK;
}

}  // namespace dmm

namespace {
// the plan with its op list written out, or null
const dmm_plan_t *listed(const dmm_plan_t *p) {
  if (!p) return nullptr;
  return dmm::materialize(const_cast<dmm_plan_t *>(p)) == DMM_OK ? p : nullptr;
}
}  // namespace

extern "C" {

int dmm_plan(const dmm_matrix_desc *A, const dmm_matrix_desc *B, const dmm_matrix_desc *C, int32_t nranks,
             uint32_t flags, dmm_plan_t **out) {
  if (!A || !B || !C || !out || nranks < 1) return DMM_EINVAL;
  if (flags & ~(DMM_STATIONARY_B | DMM_STATIONARY_A | DMM_ITERATION_OFFSET | DMM_MERGE_ALWAYS)) return DMM_EINVAL;
  if ((flags & DMM_STATIONARY_B) && (flags & DMM_STATIONARY_A)) return DMM_EINVAL;
  dmm_plan_t *P = new (std::nothrow) dmm_plan_t;
  if (!P) return DMM_ENOMEM;
  int rc = DMM_OK;
  try {
    P->nranks = nranks;
    if ((rc = dmm::load_grid(A, nranks, &P->A)) || (rc = dmm::load_grid(B, nranks, &P->B)) ||
        (rc = dmm::load_grid(C, nranks, &P->C))) {
      delete P;
      return rc;
    }
    if (P->A.cols != P->B.rows || P->A.rows != P->C.rows || P->B.cols != P->C.cols) {
      delete P;
      return DMM_ESHAPE;
    }
    P->flags = flags;
    dmm::build_merged(P, flags);
    // With a merged work list the op list is not needed to run the plan: it is written out when
    // somebody asks for it (an accessor, or dmm_execute when it has to run the other list).
    if (!P->merged.valid && (rc = dmm::materialize(P))) {
      delete P;
      return rc;
    }
  } catch (const std::bad_alloc &) {
    delete P;
    return DMM_ENOMEM;
  }
  *out = P;
  return DMM_OK;
}

int64_t dmm_plan_num_tasks(const dmm_plan_t *p) { return (p = listed(p)) ? (int64_t)p->tasks.size() : 0; }
const dmm_task *dmm_plan_tasks(const dmm_plan_t *p) { return (p = listed(p)) ? p->tasks.data() : nullptr; }
const int64_t *dmm_plan_order(const dmm_plan_t *p) { return (p = listed(p)) ? p->order.data() : nullptr; }
int64_t dmm_plan_num_groups(const dmm_plan_t *p) { return (p = listed(p)) ? (int64_t)p->groups.size() : 0; }
const int64_t *dmm_plan_group_offsets(const dmm_plan_t *p) { return (p = listed(p)) ? p->group_offsets.data() : nullptr; }
int64_t dmm_plan_num_items(const dmm_plan_t *p) { return (p = listed(p)) ? (int64_t)p->items.size() : 0; }
const dmm_work_item *dmm_plan_items(const dmm_plan_t *p) { return (p = listed(p)) ? p->items.data() : nullptr; }
int32_t dmm_plan_macro_tile(const dmm_plan_t *) { return dmm::kMacroTile; }
int64_t dmm_plan_num_merged_items(const dmm_plan_t *p) { return p && p->merged.valid ? (int64_t)p->merged.view.size() : 0; }
const dmm_merged_item *dmm_plan_merged_items(const dmm_plan_t *p) {
  return p && p->merged.valid ? p->merged.view.data() : nullptr;
}

void dmm_plan_destroy(dmm_plan_t *p) {
  if (!p) return;
  if (p->dev) dmm::destroy_device_state(p->dev);
  delete p;
}

const char *dmm_strerror(int status) {
  switch (status) {
    case DMM_OK: return "ok";
    case DMM_EINVAL: return "invalid argument (null pointer, bad cut points, empty grid, bad dtype or flag)";
    case DMM_ESHAPE: return "shapes do not form C[m,n] = A[m,k] B[k,n]";
    case DMM_EREPL: return "replication factor does not divide the rank count, or process grid too large for one replica";
    case DMM_ENOMEM: return "out of memory";
    case DMM_EHIP: return "a HIP call failed (see dmm_last_hip_error)";
    case DMM_ELD: return "leading dimension smaller than the tile width";
    case DMM_ELIMIT: return "work tables larger than the library's static device buffer";
    default: return "unknown status";
  }
}

int dmm_version(void) { return 4; }

}  // extern "C"
