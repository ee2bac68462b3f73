// Device-facing half of the library (gfx950 only): the entry points that turn a plan plus
// tile pointers into device work tables and launch the grouped GEMM (gemm_kernel.hpp), the
// replica sum, the replica broadcast and the measurement aids (aux_kernels.hpp), on top of the
// pools and the uploader of device_state.hpp.
#include <hip/hip_runtime.h>
#include <rocprofiler-sdk-roctx/roctx.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <utility>
#include <vector>

#include "aux_kernels.hpp"
#include "device_state.hpp"
#include "gemm_kernel.hpp"
#include "gemm_launch.hpp"
#include "plan_internal.h"

namespace dmm {

namespace {

static_assert(kMaxPieces == PMAX && kDescBytes == DESC_LDS - DESC_GEO && sizeof(PieceDev) == 24 &&
                  kPieceAlign * 2 >= 16 && 2 * (PMAX + 1) * 4 <= 128 && 128 + PMAX * PMAX * 24 <= DESC_GEO && kMacroTile == BM && kMacroTile == BN,
              "the planner's limits for merged macro-tiles describe the kernel's descriptor area");

// A named range on the calling thread for tracing tools (rocprofv3 --marker-trace), closed when
// the object goes out of scope: "dmm_execute" with "tables" (host assembly of the work tables and
// their upload), "gemm" and "replica_sum" (the launches) inside it, "dmm_reduce_replicas", ...
struct TraceRange {
  explicit TraceRange(const char *name) { roctxRangePushA(name); }
  ~TraceRange() { end(); }
  void end() {                        // (ranges nest: end them in reverse order of their construction)
    if (open_) roctxRangePop();
    open_ = false;
  }
  TraceRange(const TraceRange &) = delete;
  TraceRange &operator=(const TraceRange &) = delete;

 private:
  bool open_ = true;
};

// Whether the current device lets one workgroup have the stages plus the descriptor area (the
// merged macro-tile kernels); decided in ensure_state.
bool g_comp_ok[64] = {};

int ensure_state(dmm_plan_t *P) {
  // the kernels' LDS size has to be allowed once per device
  static std::mutex mu;
  static bool done[64] = {};
  int device = 0;
  DMM_HIP(hipGetDevice(&device));
  if (device < 0 || device >= 64) return DMM_EINVAL;
  {
    std::lock_guard<std::mutex> g(mu);
    if (!done[device]) {
      DMM_HIP(gemm_allow_lds_0());
      DMM_HIP(gemm_allow_lds_1());
      DMM_HIP(gemm_allow_lds_2());
      DMM_HIP(gemm_allow_lds_3());
      const bool ok = gemm_allow_lds_4() == hipSuccess && gemm_allow_lds_5() == hipSuccess;
      if (!ok) (void)hipGetLastError();
      g_comp_ok[device] = ok;
      done[device] = true;
    }
  }
  if (!P->dev) {
    P->dev = new (std::nothrow) DeviceState;
    if (!P->dev) return DMM_ENOMEM;
    DMM_HIP(hipEventCreateWithFlags(&P->dev->last_use, hipEventDisableTiming));
  }
  return DMM_OK;
}

// Compute units of the current device (queried once per device).
int device_cus(int *out) {
  static std::mutex mu;
  static int cus[64] = {};
  int dev = 0;
  DMM_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return DMM_EINVAL;
  std::lock_guard<std::mutex> g(mu);
  if (!cus[dev]) {
    hipDeviceProp_t prop;
    DMM_HIP(hipGetDeviceProperties(&prop, dev));
    cus[dev] = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 1;
  }
  *out = cus[dev];
  return DMM_OK;
}

// Event after which the kernels of this plan's earlier calls have finished (null: none yet).
hipEvent_t busy_event(dmm_plan_t *P) { return P->dev->last_use_recorded ? P->dev->last_use : nullptr; }

int mark_use(dmm_plan_t *P, hipStream_t stream) {
  DMM_HIP(hipEventRecord(P->dev->last_use, stream));
  P->dev->last_use_recorded = true;
  return DMM_OK;
}

int timing_events(hipEvent_t ev[2]) {
  for (int i = 0; i < 2; ++i)
    if (!ev[i]) DMM_HIP(hipEventCreate(&ev[i]));
  return DMM_OK;
}

// ld >= width for every non-empty tile of a matrix
int check_lds(const Grid &G, const int64_t *ld) {
  for (int32_t rep = 0; rep < G.c; ++rep)
    for (int32_t ti = 0; ti < G.gr; ++ti)
      for (int32_t tj = 0; tj < G.gc; ++tj) {
        const int64_t w = G.cc[tj + 1] - G.cc[tj], h = G.rc[ti + 1] - G.rc[ti];
        if (w > 0 && h > 0 && ld[G.table_index(rep, ti, tj)] < w) return DMM_ELD;
      }
  return DMM_OK;
}

// The replica sum in two halves, so that dmm_execute can put the table upload in front of the
// GEMM launch and nothing but the launch itself behind it.
// Appends the replica sum's tables to *h at byte offset `base` (a multiple of 8).
int build_reduce(dmm_plan_t *P, void *const *c_tiles, const int64_t *c_ld, int32_t origin, std::vector<char> *hp,
                 size_t base, RedLaunch *L) {
  const Grid &C = P->C;
  L->n_items = 0;
  if (C.c <= 1) return DMM_OK;
  const int nparts = C.c;
  std::vector<RedTile> tiles;
  std::vector<RedItem> items;
  std::vector<const float *> parts;
  std::vector<int64_t> part_ld;
  bool vec_ok = true;
  for (int32_t ti = 0; ti < C.gr; ++ti)
    for (int32_t tj = 0; tj < C.gc; ++tj) {
      const int64_t rows = C.rc[ti + 1] - C.rc[ti], cols = C.cc[tj + 1] - C.cc[tj];
      if (rows <= 0 || cols <= 0) continue;
      RedTile t;
      const int64_t oi = C.table_index(origin, ti, tj);
      t.out = (float *)c_tiles[oi];
      t.ldo = c_ld[oi];
      t.part_begin = (int64_t)parts.size();
      t.rows = (int32_t)rows;
      t.cols = (int32_t)cols;
      if (!t.out) return DMM_EINVAL;
      if (((uintptr_t)t.out & 15) || (t.ldo & 3) || (cols & 3)) vec_ok = false;
      for (int32_t rep = 0; rep < nparts; ++rep) {
        const int64_t pi = C.table_index(rep, ti, tj);
        const float *pp = (const float *)c_tiles[pi];
        if (!pp) return DMM_EINVAL;
        if (((uintptr_t)pp & 15) || (c_ld[pi] & 3)) vec_ok = false;
        parts.push_back(pp);
        part_ld.push_back(c_ld[pi]);
      }
      // blocks of rows holding about RED_ELEMS elements each
      int64_t per = (RED_ELEMS + cols - 1) / cols;
      if (per < 1) per = 1;
      for (int64_t r = 0; r < rows; r += per) {
        RedItem it;
        it.tile = (int32_t)tiles.size();
        it.row0 = (int32_t)r;
        it.nrows = (int32_t)(rows - r < per ? rows - r : per);
        it.pad = 0;
        items.push_back(it);
      }
      tiles.push_back(t);
    }
  if (items.empty()) return DMM_OK;
  // items | tiles | part pointers | part lds   (all 8-byte aligned)
  const size_t o_items = base;
  const size_t o_tiles = o_items + items.size() * sizeof(RedItem);
  const size_t o_parts = o_tiles + tiles.size() * sizeof(RedTile);
  const size_t o_lds = o_parts + parts.size() * sizeof(void *);
  const size_t total = o_lds + part_ld.size() * sizeof(int64_t);
  std::vector<char> &h = *hp;
  h.resize(total);
  std::memcpy(h.data() + o_items, items.data(), items.size() * sizeof(RedItem));
  std::memcpy(h.data() + o_tiles, tiles.data(), tiles.size() * sizeof(RedTile));
  std::memcpy(h.data() + o_parts, parts.data(), parts.size() * sizeof(void *));
  std::memcpy(h.data() + o_lds, part_ld.data(), part_ld.size() * sizeof(int64_t));
  L->n_items = items.size();
  L->o_items = o_items;
  L->o_tiles = o_tiles;
  L->o_parts = o_parts;
  L->o_lds = o_lds;
  L->nparts = nparts;
  L->vec_ok = vec_ok;
  return DMM_OK;
}

// The replica sum's (or the broadcast's) tables alone, uploaded through the plan's second buffer.
int stage_reduce(dmm_plan_t *P, void *const *c_tiles, const int64_t *c_ld, int32_t origin, hipStream_t stream,
                 RedLaunch *L) {
  std::vector<char> &h = P->dev->host;
  h.clear();
  int rc = build_reduce(P, c_tiles, c_ld, origin, &h, 0, L);
  if (rc || L->n_items == 0) return rc;
  if ((rc = P->dev->red_table.upload(h.data(), h.size(), stream, busy_event(P)))) return rc;
  L->dev_base = P->dev->red_table.dev();
  return DMM_OK;
}

int fire_reduce(dmm_plan_t *P, const RedLaunch &L, hipStream_t stream, bool timed) {
  if (L.n_items == 0) return DMM_OK;
  int rc;
  char *d = L.dev_base;
  const size_t o_items = L.o_items, o_tiles = L.o_tiles, o_parts = L.o_parts, o_lds = L.o_lds;
  const int nparts = L.nparts;
  const bool vec_ok = L.vec_ok;
  if (timed) {
    if ((rc = timing_events(P->dev->t_red))) return rc;
    DMM_HIP(hipEventRecord(P->dev->t_red[0], stream));
  }
  hipLaunchKernelGGL(reduce_replicas_kernel, dim3((unsigned)L.n_items), dim3(RED_NT), 0, stream,
                     (const RedItem *)(d + o_items), (const RedTile *)(d + o_tiles),
                     (const float *const *)(d + o_parts), (const int64_t *)(d + o_lds), nparts, vec_ok ? 1 : 0);
  DMM_HIP(hipGetLastError());
  if (timed) {
    DMM_HIP(hipEventRecord(P->dev->t_red[1], stream));
    P->dev->red_timed = true;
  }
  return DMM_OK;
}

// Device tables of the merged macro-tiles, appended to *hp (empty on entry):
//   CompItemDev[items] | PieceDev a[...] | PieceDev b[...] | PieceDev c[...] | int32 klen[...]
// A slices are numbered (replica, row interval, segment), B slices (replica, segment, column
// interval), C slices (replica, row interval, column interval).
// K steps a run of a macro-tile cut along K has at least (see build_group_exec): 64 with bf16
// operands, measured; a K step of fp32 operands keeps the matrix pipes busy eight times as long
// (128 MFMAs of 64 cycles against 32 of 32), so there a run of the same duration is 8 steps.
constexpr int32_t MIN_RUN = 64;
inline int32_t min_run_steps(int64_t es) { return es == 4 ? MIN_RUN / 8 : MIN_RUN; }

// Scratch buffer of the plan for `n_runs` partial tiles; orders this call behind the plan's last one.
int acquire_split_buffer(dmm_plan_t *P, size_t n_runs, hipStream_t stream) {
  // the scratch buffer is shared by all calls on this plan: order this call behind the last one
  // (a no-op when both are on the same stream)
  if (P->dev->last_use_recorded) DMM_HIP(hipStreamWaitEvent(stream, P->dev->last_use, 0));
  const size_t need = n_runs * sizeof(float) * BM * BN;
  if (need > P->dev->split_cap) {
    // growing: earlier calls on this plan may still use the old buffer
    if (P->dev->split_buf) {
      DMM_HIP(hipStreamSynchronize(stream));
      scratch_pool().release(&P->dev->split_buf, &P->dev->split_cap);
    }
    return scratch_pool().acquire(need, &P->dev->split_buf, &P->dev->split_cap);
  }
  return DMM_OK;
}

int build_merged_tables(dmm_plan_t *P, int64_t es, int64_t bk, int64_t c_es, const void *const *a_tiles,
                        const int64_t *a_ld, const void *const *b_tiles, const int64_t *b_ld, void *const *c_tiles,
                        const int64_t *c_ld, int cus, hipStream_t stream, std::vector<char> *hp, MergedLaunch *L) {
  const Merged &G = P->merged;
  const Grid &A = P->A, &B = P->B, &C = P->C;
  const size_t MR = G.mc.size() - 1, NR = G.nc.size() - 1;
  // tile that holds a cut point (the last tile whose lower cut is not above it: skips empty tiles)
  auto holder = [](const std::vector<int64_t> &cuts, int64_t x) {
    return (int32_t)(std::upper_bound(cuts.begin(), cuts.end() - 1, x) - cuts.begin()) - 1;
  };
  std::vector<int32_t> a_ti(MR), c_ti(MR), b_tj(NR), c_tj(NR);
  for (size_t i = 0; i < MR; ++i) { a_ti[i] = holder(A.rc, G.mc[i]); c_ti[i] = holder(C.rc, G.mc[i]); }
  for (size_t j = 0; j < NR; ++j) { b_tj[j] = holder(B.cc, G.nc[j]); c_tj[j] = holder(C.cc, G.nc[j]); }
  std::vector<PieceDev> pa, pb, pc;
  std::vector<int32_t> klen;
  std::vector<int32_t> a0(G.reps.size()), b0(G.reps.size()), c0(G.reps.size()), k0(G.reps.size()), steps(G.reps.size());
  std::vector<std::vector<int32_t>> steps_before(G.reps.size());   // K steps in front of every segment, per replica
  auto piece = [](const void *base, int64_t ld, int64_t r, int64_t c, int64_t h, int64_t w, int64_t esz) {
    PieceDev d;
    const int64_t off = r * ld + c;
    d.ptr = (const char *)base + off * esz;
    d.room = ((h - 1) * ld + w - off) * esz;
    d.pitch = (uint32_t)(ld * esz);
    d.pad = 0;
    return d;
  };
  for (size_t rep = 0; rep < G.reps.size(); ++rep) {
    const MergedRep &R = G.reps[rep];
    const size_t S = R.kc.size() - 1;
    a0[rep] = (int32_t)pa.size();
    b0[rep] = (int32_t)pb.size();
    c0[rep] = (int32_t)pc.size();
    k0[rep] = (int32_t)klen.size();
    std::vector<int32_t> a_tj(S), b_ti(S);
    int32_t nsteps = 0;
    for (size_t s = 0; s < S; ++s) {
      a_tj[s] = holder(A.cc, R.kc[s]);
      b_ti[s] = holder(B.rc, R.kc[s]);
      klen.push_back((int32_t)(R.kc[s + 1] - R.kc[s]));
      steps_before[rep].push_back(nsteps);
      nsteps += (int32_t)((R.kc[s + 1] - R.kc[s] + bk - 1) / bk);
    }
    steps_before[rep].push_back(nsteps);
    steps[rep] = nsteps;
    for (size_t i = 0; i < MR; ++i)
      for (size_t s = 0; s < S; ++s) {
        const int32_t ti = a_ti[i], tj = a_tj[s];
        const int64_t idx = A.table_index(R.a_rep, ti, tj);
        if (!a_tiles[idx]) return DMM_EINVAL;
        pa.push_back(piece(a_tiles[idx], a_ld[idx], G.mc[i] - A.rc[ti], R.kc[s] - A.cc[tj], A.rc[ti + 1] - A.rc[ti],
                           A.cc[tj + 1] - A.cc[tj], es));
      }
    for (size_t s = 0; s < S; ++s)
      for (size_t j = 0; j < NR; ++j) {
        const int32_t ti = b_ti[s], tj = b_tj[j];
        const int64_t idx = B.table_index(R.b_rep, ti, tj);
        if (!b_tiles[idx]) return DMM_EINVAL;
        pb.push_back(piece(b_tiles[idx], b_ld[idx], R.kc[s] - B.rc[ti], G.nc[j] - B.cc[tj], B.rc[ti + 1] - B.rc[ti],
                           B.cc[tj + 1] - B.cc[tj], es));
      }
    for (size_t i = 0; i < MR; ++i)
      for (size_t j = 0; j < NR; ++j) {
        const int32_t ti = c_ti[i], tj = c_tj[j];
        const int64_t idx = C.table_index((int32_t)rep, ti, tj);
        if (!c_tiles[idx]) return DMM_EINVAL;
        pc.push_back(piece(c_tiles[idx], c_ld[idx], G.mc[i] - C.rc[ti], G.nc[j] - C.cc[tj], C.rc[ti + 1] - C.rc[ti],
                           C.cc[tj + 1] - C.cc[tj], c_es));
      }
  }
  std::vector<CompItemDev> items(G.items.size());
  for (size_t x = 0; x < G.items.size(); ++x) {
    const MergedItem &w = G.items[x];
    const size_t S = G.reps[(size_t)w.rep].kc.size() - 1;
    CompItemDev d;
    std::memset(&d, 0, sizeof(d));
    d.m_ext = w.m_ext;
    d.n_ext = w.n_ext;
    d.R = w.R;
    d.Q = w.Q;
    d.S = (int32_t)S;
    d.nsteps = steps[(size_t)w.rep];
    d.c_es = (int32_t)c_es;
    d.a_first = a0[(size_t)w.rep] + w.mr0 * (int32_t)S;
    d.a_stride = (int32_t)S;
    d.b_first = b0[(size_t)w.rep] + w.nr0;
    d.b_stride = (int32_t)NR;
    d.c_first = c0[(size_t)w.rep] + w.mr0 * (int32_t)NR + w.nr0;
    d.c_stride = (int32_t)NR;
    d.k_first = k0[(size_t)w.rep];
    for (int32_t p = 0; p <= w.R; ++p) d.rb[p] = (int32_t)(G.mc[(size_t)(w.mr0 + p)] - w.m0);
    for (int32_t q = 0; q <= w.Q; ++q) d.cb[q] = (int32_t)(G.nc[(size_t)(w.nr0 + q)] - w.n0);
    items[x] = d;
  }
  // K-split of the last round, as for the per-group macro-tiles: the last W % cus macro-tiles, if
  // they are at most half a round, are cut into runs of at least min_run_steps() K steps; every run writes
  // a plain partial tile to the scratch buffer, and the partial tiles of a macro-tile are added up
  // piece by piece (one FixItem per row piece and column piece, each with its own C slice).
  std::vector<FixItem> fixes;
  size_t n_runs = 0;
  const size_t n_whole = items.size();
  // one FixItem per (row piece, column piece) of a macro-tile whose `runs` partial tiles start at
  // partial tile number `first_part`
  auto fix_pieces = [&](const CompItemDev &whole, size_t first_part, int32_t runs) {
    for (int32_t p = 0; p < whole.R; ++p)
      for (int32_t q = 0; q < whole.Q; ++q) {
        const int32_t r0 = std::max(whole.rb[p], 0), r1 = std::min(whole.rb[p + 1], whole.m_ext);
        const int32_t q0 = std::max(whole.cb[q], 0), q1 = std::min(whole.cb[q + 1], whole.n_ext);
        const PieceDev &cp = pc[(size_t)(whole.c_first + p * whole.c_stride + q)];
        FixItem f;
        f.dst = (void *)(cp.ptr + (int64_t)(r0 - whole.rb[p]) * cp.pitch + (int64_t)(q0 - whole.cb[q]) * c_es);
        f.ldc = (int64_t)cp.pitch / c_es;
        f.parts = (const float *)(uintptr_t)(first_part * sizeof(float) * BM * BN);   // offset for now
        f.m_ext = r1 - r0;
        f.n_ext = q1 - q0;
        f.nparts = runs;
        f.c_es = (int32_t)c_es;
        f.row0 = r0;
        f.col0 = q0;
        fixes.push_back(f);
      }
  };
  // Cutting macro-tiles along K.  Two reasons, one mechanism: (a) the plan asks for it (G.window:
  // the descriptors of all of a macro-tile's segments would not fit beside eight pieces per axis),
  // (b) the macro-tiles fill the device badly: at most half a round of them in all, or a last round
  // that is at most half full (then its macro-tiles only), as for the per-group macro-tiles.  A run
  // is a range of at least min_run_steps() K steps; its workgroup stages the descriptors of the segments
  // the range touches only, starts `first_step` steps into the first of them and writes a plain
  // partial tile.  Launch order: the first run of every macro-tile in the macro-tiles' own order,
  // then the second of every one, ...
  auto desc_bytes = [](int64_t segs, int64_t pieces) { return 4 * ((segs + 3) & ~(int64_t)3) + 24 * segs * pieces; };
  std::vector<int32_t> want(n_whole, 1);                 // runs wanted per macro-tile
  size_t total = 0;
  for (size_t x = 0; x < n_whole; ++x) {
    if (G.window > 0 && items[x].S > G.window) want[x] = (items[x].S + G.window - 1) / G.window;
    total += (size_t)want[x];
  }
  if (total <= (size_t)cus / 2) {
    const int32_t f = (int32_t)((size_t)cus / total);
    for (size_t x = 0; x < n_whole; ++x) want[x] *= f;
  } else if (G.window == 0) {
    const size_t tail = n_whole % (size_t)cus;
    if (tail > 0 && tail <= (size_t)cus / 2)
      for (size_t x = n_whole - tail; x < n_whole; ++x) want[x] = (int32_t)((size_t)cus / tail);
  }
  std::vector<CompItemDev> later;
  for (size_t x = 0; x < n_whole; ++x) {
    const CompItemDev whole = items[x];
    const std::vector<int32_t> &before = steps_before[(size_t)G.items[x].rep];
    const int32_t least = G.window > 0 && whole.S > G.window ? (whole.S + G.window - 1) / G.window : 1;
    int32_t runs = std::max(least, std::min(want[x], whole.nsteps / min_run_steps(es)));
    if (runs < 2) continue;
    // ranges of `per` steps; more runs if some range touches more segments than fit
    int32_t per = 0;
    for (;; ++runs) {
      per = (whole.nsteps + runs - 1) / runs;
      bool fits = true;
      for (int32_t t0 = 0; t0 < whole.nsteps && fits; t0 += per) {
        const int32_t t1 = std::min(t0 + per, whole.nsteps);
        const int64_t lo = std::upper_bound(before.begin(), before.end(), t0) - before.begin() - 1;
        const int64_t hi = std::upper_bound(before.begin(), before.end(), t1 - 1) - before.begin() - 1;
        fits = desc_bytes(hi - lo + 1, whole.R + whole.Q) <= kDescBytes;
      }
      if (fits || per == 1) break;
    }
    runs = (whole.nsteps + per - 1) / per;
    if (runs < 2) continue;
    fix_pieces(whole, n_runs, runs);
    for (int32_t j = 0; j < runs; ++j) {
      const int32_t t0 = j * per, t1 = std::min(t0 + per, whole.nsteps);
      const int32_t lo = (int32_t)(std::upper_bound(before.begin(), before.end(), t0) - before.begin()) - 1;
      const int32_t hi = (int32_t)(std::upper_bound(before.begin(), before.end(), t1 - 1) - before.begin()) - 1;
      CompItemDev r = whole;
      r.S = hi - lo + 1;
      r.a_first = whole.a_first + lo;
      r.b_first = whole.b_first + lo * whole.b_stride;
      r.k_first = whole.k_first + lo;
      r.first_step = t0 - before[(size_t)lo];
      r.nsteps = t1 - t0;
      r.scratch = (float *)(uintptr_t)((n_runs + (size_t)j) * sizeof(float) * BM * BN);   // offset for now
      r.pad = 1 + j;                                                                        // marks the offset; run number + 1
      if (j == 0) items[x] = r;
      else later.push_back(r);
    }
    n_runs += (size_t)runs;
  }
  std::stable_sort(later.begin(), later.end(), [](const CompItemDev &a, const CompItemDev &b) { return a.pad < b.pad; });
  for (CompItemDev &r : later) r.pad = 1;
  for (CompItemDev &r : items)
    if (r.pad > 0) r.pad = 1;
  items.insert(items.end(), later.begin(), later.end());
  if (n_runs > 0) {
    int rc = acquire_split_buffer(P, n_runs, stream);
    if (rc) return rc;
    for (CompItemDev &d : items)
      if (d.pad == 1) {
        d.scratch = (float *)(P->dev->split_buf + (uintptr_t)d.scratch);
        d.pad = 0;
      }
    for (FixItem &f : fixes) f.parts = (const float *)(P->dev->split_buf + (uintptr_t)f.parts);
  }
  L->n_items = items.size();
  L->n_fix = fixes.size();
  L->o_a = items.size() * sizeof(CompItemDev);
  L->o_b = L->o_a + pa.size() * sizeof(PieceDev);
  L->o_c = L->o_b + pb.size() * sizeof(PieceDev);
  L->o_k = L->o_c + pc.size() * sizeof(PieceDev);
  L->o_fix = (L->o_k + klen.size() * sizeof(int32_t) + 7) & ~(size_t)7;
  L->total = L->o_fix + fixes.size() * sizeof(FixItem);
  std::vector<char> &h = *hp;
  h.assign(L->total, 0);
  std::memcpy(h.data(), items.data(), items.size() * sizeof(CompItemDev));
  std::memcpy(h.data() + L->o_a, pa.data(), pa.size() * sizeof(PieceDev));
  std::memcpy(h.data() + L->o_b, pb.data(), pb.size() * sizeof(PieceDev));
  std::memcpy(h.data() + L->o_c, pc.data(), pc.size() * sizeof(PieceDev));
  std::memcpy(h.data() + L->o_k, klen.data(), klen.size() * sizeof(int32_t));
  if (!fixes.empty()) std::memcpy(h.data() + L->o_fix, fixes.data(), fixes.size() * sizeof(FixItem));
  return DMM_OK;
}

}  // namespace
}  // namespace dmm

extern "C" {

int dmm_last_hip_error(void) { return dmm::g_last_hip_error; }

int dmm_measure_mfma_rate(float milliseconds, int random_operands, float *tflops, float *shader_mhz) {
  using namespace dmm;
  if (!(milliseconds > 0.f) || milliseconds > 1000.f) return DMM_EINVAL;
  int dev = 0;
  hipDeviceProp_t prop;
  DMM_HIP(hipGetDevice(&dev));
  DMM_HIP(hipGetDeviceProperties(&prop, dev));
  const int blocks = prop.multiProcessorCount;      // one block of four waves per CU
  unsigned long long *d_cycles = nullptr;
  float *d_sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = DMM_OK;
  auto fail = [&](hipError_t e) {
    if (e != hipSuccess && rc == DMM_OK) {
      g_last_hip_error = (int)e;
      rc = DMM_EHIP;
    }
    return e != hipSuccess;
  };
  std::vector<unsigned long long> h((size_t)blocks);
  float ms = 0.f;
  double cyc = 0.0;
  int iters = 4000;                                 // first pass: ~1 ms, to size the second
  if (fail(hipMalloc((void **)&d_cycles, sizeof(unsigned long long) * (size_t)blocks))) goto done;
  if (fail(hipMalloc((void **)&d_sink, sizeof(float)))) goto done;
  if (fail(hipEventCreate(&e0)) || fail(hipEventCreate(&e1))) goto done;
  for (int pass = 0; pass < 2; ++pass) {
    if (fail(hipEventRecord(e0, nullptr))) goto done;
    hipLaunchKernelGGL(mfma_rate_kernel, dim3((unsigned)blocks), dim3(256), 0, nullptr, d_cycles, d_sink, iters,
                       random_operands);
    if (fail(hipGetLastError())) goto done;
    if (fail(hipEventRecord(e1, nullptr)) || fail(hipEventSynchronize(e1))) goto done;
    if (fail(hipEventElapsedTime(&ms, e0, e1))) goto done;
    if (pass == 0) {
      double scale = (double)milliseconds / (ms > 1e-3f ? ms : 1e-3f);
      double want = iters * scale;
      if (want > 2.0e8) want = 2.0e8;
      iters = (int)(want / 4) * 4;
      if (iters < 4) iters = 4;
    }
  }
  if (fail(hipMemcpy(h.data(), d_cycles, sizeof(unsigned long long) * (size_t)blocks, hipMemcpyDeviceToHost))) goto done;
  for (unsigned long long c : h) cyc += (double)c;
  cyc /= blocks;
  // per block: 4 waves x iters x 8 MFMAs x 32 * 32 * 16 * 2 flop
  if (tflops) *tflops = (float)((double)blocks * 4.0 * iters * 8.0 * 32768.0 / (ms * 1e-3) / 1e12);
  if (shader_mhz) *shader_mhz = (float)(cyc / (ms * 1e-3) / 1e6);
done:
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (d_cycles) (void)hipFree(d_cycles);
  if (d_sink) (void)hipFree(d_sink);
  return rc;
}

namespace dmm {
namespace {

struct ExecArgs {
  int dtype;
  int64_t es, bk, c_es;
  const void *const *a_tiles;
  const int64_t *a_ld;
  const void *const *b_tiles;
  const int64_t *b_ld;
  void *const *c_tiles;
  const int64_t *c_ld;
  uint32_t flags;
  int device;
};

// Work tables of the merged macro-tiles:  merged tables | replica-sum tables, one copy.
int build_merged_exec(dmm_plan_t *P, const ExecArgs &x, hipStream_t stream, ExecLayout *L) {
  int rc;
  RedLaunch red;
  MergedLaunch ml;
  std::vector<char> &h = P->dev->host;
  h.clear();
  int cus = 0;
  if ((rc = device_cus(&cus))) return rc;
  if ((rc = build_merged_tables(P, x.es, x.bk, x.c_es, x.a_tiles, x.a_ld, x.b_tiles, x.b_ld, x.c_tiles, x.c_ld, cus, stream, &h, &ml)))
    return rc;
  if (!(x.flags & DMM_NO_REDUCE) && (rc = build_reduce(P, x.c_tiles, x.c_ld, 0, &h, ml.total, &red))) return rc;
  if ((rc = P->dev->gemm_table.upload(h.data(), h.size(), stream, busy_event(P)))) return rc;
  red.dev_base = P->dev->gemm_table.dev();
  L->merged = true;
  L->ml = ml;
  L->red = red;
  L->uses_split = ml.n_fix > 0;
  return DMM_OK;
}

// Work tables of the per-group macro-tiles.  The tables of all kernels go up in one copy in front
// of the GEMM launch, so that nothing but the launches separates them:
// ItemDev[] | SegDev[] | FixItem[] | RedSrc[] | replica-sum tables.
int build_group_exec(dmm_plan_t *P, const ExecArgs &x, hipStream_t stream, ExecLayout *L) {
  int rc;
  const int64_t es = x.es, bk = x.bk, c_es = x.c_es;
  const void *const *a_tiles = x.a_tiles;
  const void *const *b_tiles = x.b_tiles;
  void *const *c_tiles = x.c_tiles;
  const int64_t *a_ld = x.a_ld, *b_ld = x.b_ld, *c_ld = x.c_ld;
  const uint32_t flags = x.flags;
  if ((rc = materialize(P))) return rc;
    RedLaunch red;
  const size_t n_plan_items = P->items.size();
  const size_t n_segs = P->tasks.size();
  std::vector<SegDev> hs(n_segs);
  std::vector<ItemDev> hi(n_plan_items);
  std::vector<FixItem> fixes;
  // segments in grouped order: segment index = position in `order`
  for (size_t pos = 0; pos < n_segs; ++pos) {
    const dmm_task &t = P->tasks[P->order[pos]];
    const int64_t ai = P->A.table_index(t.a_rep, t.a_ti, t.a_tj);
    const int64_t bi = P->B.table_index(t.b_rep, t.b_ti, t.b_tj);
    if (!a_tiles[ai] || !b_tiles[bi]) return DMM_EINVAL;
    SegDev sg;
    sg.lda = a_ld[ai];
    sg.ldb = b_ld[bi];
    sg.a = (const char *)a_tiles[ai] + ((t.m0 - P->A.rc[t.a_ti]) * sg.lda + (t.k0 - P->A.cc[t.a_tj])) * es;
    sg.b = (const char *)b_tiles[bi] + ((t.k0 - P->B.rc[t.b_ti]) * sg.ldb + (t.n0 - P->B.cc[t.b_tj])) * es;
    // bytes that may be read from the segment's origin to the end of the tile buffer
    // ((rows - 1) * ld + cols elements are guaranteed to exist)
    const int64_t a_h = P->A.rc[t.a_ti + 1] - P->A.rc[t.a_ti], a_w = P->A.cc[t.a_tj + 1] - P->A.cc[t.a_tj];
    const int64_t b_h = P->B.rc[t.b_ti + 1] - P->B.rc[t.b_ti], b_w = P->B.cc[t.b_tj + 1] - P->B.cc[t.b_tj];
    sg.a_bytes = ((a_h - 1) * sg.lda + a_w - ((t.m0 - P->A.rc[t.a_ti]) * sg.lda + (t.k0 - P->A.cc[t.a_tj]))) * es;
    sg.b_bytes = ((b_h - 1) * sg.ldb + b_w - ((t.k0 - P->B.rc[t.b_ti]) * sg.ldb + (t.n0 - P->B.cc[t.b_tj]))) * es;
    sg.klen = (int32_t)(t.k1 - t.k0);
    sg.pad = 0;
    hs[pos] = sg;
  }
  for (size_t i = 0; i < n_plan_items; ++i) {
    const dmm_work_item &w = P->items[i];
    const int64_t ci = P->C.table_index(w.c_rep, w.c_ti, w.c_tj);
    if (!c_tiles[ci]) return DMM_EINVAL;
    ItemDev d;
    d.ldc = c_ld[ci];
    d.c = (char *)c_tiles[ci] + ((w.m0 - P->C.rc[w.c_ti]) * d.ldc + (w.n0 - P->C.cc[w.c_tj])) * c_es;
    if (w.group >= 0) {
      const Group &G = P->groups[(size_t)w.group];
      d.seg_begin = (int32_t)G.first;
      d.nsteps = 0;
      for (int64_t q = 0; q < G.count; ++q) d.nsteps += (int32_t)((hs[(size_t)(G.first + q)].klen + bk - 1) / bk);
      d.m_off = (int32_t)(w.m0 - G.m0);
      d.n_off = (int32_t)(w.n0 - G.n0);
    } else {
      d.seg_begin = 0;
      d.nsteps = 0;
      d.m_off = d.n_off = 0;
    }
    d.m_ext = w.m_ext;
    d.n_ext = w.n_ext;
    d.first_step = 0;
    d.c_es = (int32_t)c_es;
    d.red_first = d.red_count = 0;
    hi[i] = d;
  }
  // K-split of the last round (see sum_parts_kernel): with W working items on `cus` CUs the
  // last W % cus of them run alone; if they are few, each is cut into up to cus / (W % cus) runs
  // of at least min_run_steps() K steps.  Run 0 takes the item's place in the launch order, the others
  // go to the end; all of them write to the scratch buffer.  A run pays a prologue and an
  // epilogue of its own (about 13 K steps' worth) and the pass that adds the runs up is one more
  // launch: measured with bf16 operands, runs of 32 steps lose (2048^3: 45 -> 66 us), so a run is
  // 64 steps at least (8 of fp32 operands, the same duration).
  int cus = 0;
  if ((rc = device_cus(&cus))) return rc;
  size_t working = 0;
  for (const ItemDev &d : hi) working += d.nsteps > 0;
  const size_t tail = working % (size_t)cus;
  size_t n_runs = 0;
  if (tail > 0 && tail <= (size_t)cus / 2) {
    const int32_t max_runs = (int32_t)((size_t)cus / tail);
    size_t seen = 0;
    for (size_t i = n_plan_items; i-- > 0 && seen < tail;) {
      if (hi[i].nsteps <= 0) continue;
      ++seen;
      int32_t runs = std::min(max_runs, hi[i].nsteps / min_run_steps(es));
      if (runs < 2) continue;
      const int32_t per = (hi[i].nsteps + runs - 1) / runs;
      runs = (hi[i].nsteps + per - 1) / per;
      const ItemDev whole = hi[i];
      FixItem f;
      f.dst = whole.c;
      f.ldc = whole.ldc;
      f.parts = (const float *)(uintptr_t)(n_runs * sizeof(float) * BM * BN);   // offset for now, base added below
      f.m_ext = whole.m_ext;
      f.n_ext = whole.n_ext;
      f.nparts = runs;
      f.c_es = whole.c_es;
      f.row0 = f.col0 = 0;
      fixes.push_back(f);
      for (int32_t j = 0; j < runs; ++j) {
        ItemDev r = whole;
        r.c = (void *)(uintptr_t)((n_runs + (size_t)j) * sizeof(float) * BM * BN);        // offset for now
        r.ldc = BN;
        r.first_step = j * per;
        r.nsteps = std::min(per, whole.nsteps - j * per);
        r.c_es = -4;                                                                        // fp32; negative marks "c is a scratch offset"
        if (j == 0) hi[i] = r;
        else hi.push_back(r);
      }
      n_runs += (size_t)runs;
    }
  }
  if (n_runs > 0) {
    if ((rc = acquire_split_buffer(P, n_runs, stream))) return rc;
    for (ItemDev &d : hi)
      if (d.c_es < 0) {
        d.c = (void *)(P->dev->split_buf + (uintptr_t)d.c);
        d.c_es = 4;
      }
    for (FixItem &f : fixes) f.parts = (const float *)(P->dev->split_buf + (uintptr_t)f.parts);
  }
  // Fused replica sum: the macro-tiles of replicas 1, 2, ... go first, those of replica 0 behind
  // them, and these add the others' partial sums to their own before they store.  No replica-sum
  // kernel runs.  (Not together with the K-split, whose runs store through a scratch buffer.)
  // One launch where the list can be laid out so that every macro-tile of replica 0 finds the
  // partial sums of its region written by its own workgroup earlier in the same launch (workgroup
  // w walks items w, w + grid, ... in order, and a wave reads back exactly the elements it stored
  // itself); otherwise two launches, replica 0's second (stream order: every partial sum is
  // complete by then).
  const bool fuse = !(flags & (DMM_SEPARATE_REDUCE | DMM_NO_REDUCE)) && P->C.c > 1 && n_runs == 0;
  std::vector<RedSrc> reds;
  size_t n_first = hi.size();               // items of the first launch
  bool one_launch = false;
  if (fuse) {
    std::vector<ItemDev> others, origin;
    others.reserve(hi.size());
    origin.reserve(hi.size());
    std::vector<std::vector<uint32_t>> of_rep((size_t)P->C.c);     // per replica: plan items in list order
    for (size_t i = 0; i < n_plan_items; ++i) {
      const dmm_work_item &w = P->items[i];
      of_rep[(size_t)w.c_rep].push_back((uint32_t)i);
      if (w.c_rep != 0) {
        others.push_back(hi[i]);
        continue;
      }
      ItemDev d = hi[i];
      d.red_first = (int32_t)reds.size();
      d.red_count = P->C.c - 1;
      for (int32_t r = 1; r < P->C.c; ++r) {
        const int64_t idx = P->C.table_index(r, w.c_ti, w.c_tj);
        if (!c_tiles[idx]) return DMM_EINVAL;
        RedSrc src;
        src.ld = c_ld[idx];
        src.p = (const float *)c_tiles[idx] + (w.m0 - P->C.rc[w.c_ti]) * src.ld + (w.n0 - P->C.cc[w.c_tj]);
        reds.push_back(src);
      }
      origin.push_back(d);
    }
    n_first = others.size();
    // One launch?  Every replica has to have as many macro-tiles as replica 0, the k-th of each
    // covering the region of replica 0's k-th, and that number has to be a whole number of rounds
    // of the grid: then the list can be laid out so that workgroup w (which walks positions w,
    // w + grid, ...) meets the partial sums of a region before it meets replica 0's macro-tile of it.
    const size_t grid = std::min<size_t>(n_plan_items, (size_t)cus);
    const size_t n0 = of_rep[0].size();
    one_launch = grid > 0 && n0 > 0 && n0 % grid == 0;
    for (int32_t r = 1; r < P->C.c && one_launch; ++r) {
      if (of_rep[(size_t)r].size() != n0) one_launch = false;
      for (size_t k = 0; k < n0 && one_launch; ++k) {
        const dmm_work_item &o = P->items[of_rep[0][k]], &s = P->items[of_rep[(size_t)r][k]];
        if (o.c_ti != s.c_ti || o.c_tj != s.c_tj || o.m0 != s.m0 || o.n0 != s.n0 || o.m_ext != s.m_ext || o.n_ext != s.n_ext)
          one_launch = false;
      }
    }
    if (one_launch) {
      // Chunk j = macro-tiles j grid .. (j + 1) grid - 1 of every replica (a round of the planner's
      // order: the 32 workgroups of an XCD on one block of neighbouring tiles).  Per workgroup and
      // chunk: `o` = the other replicas' macro-tiles, `s` = replica 0's, which adds their partial
      // sums.  All workgroups in step would read their partial sums at the same moments, at the
      // memory's pace with the matrix pipes idle; so the XCDs alternate between two schedules,
      //   o0 s0 o1 s1 o2 s2 ...      and      o0 o1 s0 o2 s1 ... s(last),
      // whose `s` fall into different rounds except the last (cfg4, four chunks: 2 % off the step
      // against o0 o1 o2 o3 s0 s1 s2 s3 everywhere; the first schedule everywhere: 1 % on).
      const size_t Q = n0 / grid;
      std::vector<ItemDev> laid(hi.size());
      std::vector<std::pair<bool, size_t>> seq;                      // (is s, chunk)
      for (size_t w = 0; w < grid; ++w) {
        seq.clear();
        if (((w % 8) & 1) == 0 || Q < 2) {
          for (size_t j = 0; j < Q; ++j) {
            seq.push_back({false, j});
            seq.push_back({true, j});
          }
        } else {
          seq.push_back({false, 0});
          for (size_t j = 0; j < Q; ++j) {
            if (j + 1 < Q) seq.push_back({false, j + 1});
            seq.push_back({true, j});
          }
        }
        size_t t = 0;
        for (const auto &e : seq) {
          const size_t k = e.second * grid + w;
          if (e.first) laid[(t++) * grid + w] = origin[k];
          else
            for (int32_t r = 1; r < P->C.c; ++r) laid[(t++) * grid + w] = hi[of_rep[(size_t)r][k]];
        }
      }
      hi = std::move(laid);
    } else {
      hi = std::move(others);
      hi.insert(hi.end(), origin.begin(), origin.end());
    }
  }
  const size_t n_items = hi.size();
  const size_t o_segs = n_items * sizeof(ItemDev);
  const size_t o_fix = o_segs + n_segs * sizeof(SegDev);
  const size_t o_red = o_fix + fixes.size() * sizeof(FixItem);
  const size_t total = n_items > 0 ? o_red + reds.size() * sizeof(RedSrc) : 0;
  std::vector<char> &h = P->dev->host;
  h.clear();
  h.resize(total);
  if (n_items > 0) {
    std::memcpy(h.data(), hi.data(), n_items * sizeof(ItemDev));
    std::memcpy(h.data() + o_segs, hs.data(), n_segs * sizeof(SegDev));
    if (!fixes.empty()) std::memcpy(h.data() + o_fix, fixes.data(), fixes.size() * sizeof(FixItem));
    if (!reds.empty()) std::memcpy(h.data() + o_red, reds.data(), reds.size() * sizeof(RedSrc));
  }
  if (!(flags & DMM_NO_REDUCE) && !fuse && (rc = build_reduce(P, c_tiles, c_ld, 0, &h, total, &red))) return rc;
  if (!h.empty()) {
    if ((rc = P->dev->gemm_table.upload(h.data(), h.size(), stream, busy_event(P)))) return rc;
    red.dev_base = P->dev->gemm_table.dev();
  }
  L->merged = false;
  L->n_items = n_items;
  L->o_segs = o_segs;
  L->o_fix = o_fix;
  L->o_red = o_red;
  L->n_first = n_first;
  L->n_fix = fixes.size();
  L->fuse = fuse;
  L->one_launch = one_launch;
  L->uses_split = n_runs > 0;
  L->n_runs = n_runs;
  L->red = red;
  return DMM_OK;
}

// The launches of one dmm_execute, from the device table the layout describes.
int launch_exec(dmm_plan_t *P, const ExecLayout &L, int64_t es, hipStream_t stream, bool timed) {
  int rc;
  char *d = P->dev->gemm_table.dev();
  if (L.merged) {
    const MergedLaunch &ml = L.ml;
    TraceRange gemm("gemm");
    if (timed) {
      if ((rc = timing_events(P->dev->t_gemm))) return rc;
      DMM_HIP(hipEventRecord(P->dev->t_gemm[0], stream));
    }
    launch_grouped_gemm_comp((int)es, (unsigned)ml.n_items, stream, (const CompItemDev *)d, (const PieceDev *)(d + ml.o_a),
                             (const PieceDev *)(d + ml.o_b), (const PieceDev *)(d + ml.o_c), (const int32_t *)(d + ml.o_k));
    DMM_HIP(hipGetLastError());
    if (ml.n_fix > 0) {
      hipLaunchKernelGGL(sum_parts_kernel, dim3((unsigned)(ml.n_fix * (BM / FIX_ROWS))), dim3(256), 0, stream,
                         (const FixItem *)(d + ml.o_fix));
      DMM_HIP(hipGetLastError());
    }
    if (timed) {
      DMM_HIP(hipEventRecord(P->dev->t_gemm[1], stream));
      P->dev->gemm_timed = true;
    }
    gemm.end();
    P->dev->ran_merged = true;
    P->dev->ran_k_split = ml.n_fix > 0;
    P->dev->ran_fused = 0;
  } else {
    P->dev->ran_merged = false;
    if (L.n_items > 0) {
      int cus = 0;
      if ((rc = device_cus(&cus))) return rc;
      const size_t n_items = L.n_items, n_first = L.n_first;
      const bool fuse = L.fuse, one_launch = L.one_launch;
      TraceRange gemm("gemm");
      const ItemDev *di = (const ItemDev *)d;
      const SegDev *ds = (const SegDev *)(d + L.o_segs);
      if (timed) {
        if ((rc = timing_events(P->dev->t_gemm))) return rc;
        DMM_HIP(hipEventRecord(P->dev->t_gemm[0], stream));
      }
      const RedSrc *dr = (const RedSrc *)(d + L.o_red);
      // {first item, count} per launch
      const size_t part[2][2] = {{0, one_launch ? n_items : n_first}, {n_first, one_launch ? 0 : n_items - n_first}};
      for (int l = 0; l < 2; ++l) {
        if (part[l][1] == 0) continue;
        const bool sums = fuse && (l == 1 || one_launch);   // the launch whose macro-tiles add the other replicas' partial sums
        // one workgroup per CU at most: workgroup w walks items w, w + grid, w + 2 grid, ... of its launch
        const int count = (int)part[l][1];
        launch_grouped_gemm((int)es, sums, (unsigned)std::min(count, cus), stream, di + part[l][0], ds, dr, count);
        DMM_HIP(hipGetLastError());
        if (timed && fuse && !one_launch && l == 0 && part[1][1] > 0) {
          if (!P->dev->t_mid) DMM_HIP(hipEventCreate(&P->dev->t_mid));
          DMM_HIP(hipEventRecord(P->dev->t_mid, stream));
          P->dev->mid_timed = true;
          P->dev->launch_flops[0] = P->dev->launch_flops[1] = 0.0;
          for (const dmm_task &t : P->tasks)
            P->dev->launch_flops[t.c_rep == 0 ? 1 : 0] += 2.0 * (double)(t.m1 - t.m0) * (double)(t.n1 - t.n0) * (double)(t.k1 - t.k0);
        }
      }
      if (L.n_fix > 0) {
        hipLaunchKernelGGL(sum_parts_kernel, dim3((unsigned)(L.n_fix * (BM / FIX_ROWS))), dim3(256), 0, stream,
                           (const FixItem *)(d + L.o_fix));
        DMM_HIP(hipGetLastError());
      }
      if (timed) {
        DMM_HIP(hipEventRecord(P->dev->t_gemm[1], stream));
        P->dev->gemm_timed = true;
      }
    }
    P->dev->ran_k_split = L.n_runs > 0;
    P->dev->ran_fused = !L.fuse ? 0 : L.one_launch ? 1 : 2;
  }
  {
    TraceRange tr("replica_sum");
    if ((rc = fire_reduce(P, L.red, stream, timed))) return rc;
  }
  return mark_use(P, stream);
}

}  // namespace
}  // namespace dmm

int dmm_execute(dmm_plan_t *P, int dtype, const void *const *a_tiles, const int64_t *a_ld,
                const void *const *b_tiles, const int64_t *b_ld, void *const *c_tiles, const int64_t *c_ld,
                uint32_t flags, void *hip_stream) {
  using namespace dmm;
  if (!P || !a_tiles || !a_ld || !b_tiles || !b_ld || !c_tiles || !c_ld) return DMM_EINVAL;
  if (dtype != DMM_BF16 && dtype != DMM_F32) return DMM_EINVAL;
  if (flags & ~(DMM_NO_REDUCE | DMM_TIMING | DMM_C_BF16 | DMM_NO_MERGE | DMM_SEPARATE_REDUCE)) return DMM_EINVAL;
  const bool timed = (flags & DMM_TIMING) != 0;
  // bf16 C tiles only where a tile receives a final sum: partial sums of a replicated C stay fp32
  if ((flags & DMM_C_BF16) && P->C.c != 1) return DMM_EINVAL;
  const int64_t c_es = (flags & DMM_C_BF16) ? 2 : 4;
  int rc;
  if ((rc = check_lds(P->A, a_ld)) || (rc = check_lds(P->B, b_ld)) || (rc = check_lds(P->C, c_ld))) return rc;
  const int64_t es = dtype == DMM_BF16 ? 2 : 4;
  const int64_t bk = dtype == DMM_BF16 ? Shape<2>::BK : Shape<4>::BK;
  // the kernel addresses a macro-tile's rows with 32-bit byte offsets, built as a 24-bit
  // multiply of (row, pitch): every row pitch has to stay below 2^24 bytes
  constexpr int64_t MAX_PITCH = (int64_t)1 << 24;
  for (int64_t i = 0; i < P->A.c * P->A.tiles_per_rep(); ++i)
    if (a_ld[i] * es >= MAX_PITCH) return DMM_ELD;
  for (int64_t i = 0; i < P->B.c * P->B.tiles_per_rep(); ++i)
    if (b_ld[i] * es >= MAX_PITCH) return DMM_ELD;
  for (int64_t i = 0; i < P->C.c * P->C.tiles_per_rep(); ++i)
    if (c_ld[i] * c_es >= MAX_PITCH) return DMM_ELD;
  hipStream_t stream = (hipStream_t)hip_stream;
  TraceRange whole("dmm_execute");
  try {
    if ((rc = ensure_state(P))) return rc;
    P->dev->gemm_timed = P->dev->red_timed = P->dev->mid_timed = false;
    int device = 0;
    DMM_HIP(hipGetDevice(&device));
    // The call's inputs, side by side: when they are those of the plan's last dmm_execute, the
    // device table of that call is still in place and describes this one too (DMM_TIMING changes
    // nothing in it), so the assembly of the tables and their upload are skipped.
    std::vector<char> &key = P->dev->key_scratch;
    key.clear();
    auto put = [&key](const void *p, size_t bytes) { key.insert(key.end(), (const char *)p, (const char *)p + bytes); };
    const int64_t head[3] = {dtype, (int64_t)(flags & ~DMM_TIMING), device};
    put(head, sizeof head);
    const size_t na = (size_t)(P->A.c * P->A.tiles_per_rep()), nb = (size_t)(P->B.c * P->B.tiles_per_rep()),
                 nc = (size_t)(P->C.c * P->C.tiles_per_rep());
    put(a_tiles, na * sizeof(void *));
    put(a_ld, na * sizeof(int64_t));
    put(b_tiles, nb * sizeof(void *));
    put(b_ld, nb * sizeof(int64_t));
    put(c_tiles, nc * sizeof(void *));
    put(c_ld, nc * sizeof(int64_t));
    ExecLayout L;
    if (P->dev->exec_cached && key == P->dev->exec_key) {
      L = P->dev->exec_layout;
      P->dev->table_reused = true;
      if ((rc = P->dev->gemm_table.order_behind_copy(stream))) return rc;
      // (the scratch buffer of macro-tiles cut along K is shared by all calls on this plan)
      if (L.uses_split && P->dev->last_use_recorded) DMM_HIP(hipStreamWaitEvent(stream, P->dev->last_use, 0));
    } else {
      P->dev->exec_cached = false;
      P->dev->table_reused = false;
      TraceRange tables("tables");
      const ExecArgs x = {dtype, es, bk, c_es, a_tiles, a_ld, b_tiles, b_ld, c_tiles, c_ld, flags, device};
      if (P->merged.valid && !(flags & DMM_NO_MERGE) && g_comp_ok[device]) rc = build_merged_exec(P, x, stream, &L);
      else rc = build_group_exec(P, x, stream, &L);
      if (rc) return rc;
      P->dev->exec_key = key;
      P->dev->exec_layout = L;
      P->dev->exec_cached = true;
    }
    return launch_exec(P, L, es, stream, timed);
  } catch (const std::bad_alloc &) {
    return DMM_ENOMEM;
  }
}

int dmm_plan_gemm_launch_ms(dmm_plan_t *P, float ms[2], double flops[2]) {
  using namespace dmm;
  if (!P || !ms || !flops) return DMM_EINVAL;
  ms[0] = ms[1] = -1.f;
  flops[0] = flops[1] = 0.0;
  if (!P->dev || !P->dev->gemm_timed || !P->dev->mid_timed) return DMM_OK;
  DMM_HIP(hipEventSynchronize(P->dev->t_gemm[1]));
  DMM_HIP(hipEventElapsedTime(&ms[0], P->dev->t_gemm[0], P->dev->t_mid));
  DMM_HIP(hipEventElapsedTime(&ms[1], P->dev->t_mid, P->dev->t_gemm[1]));
  flops[0] = P->dev->launch_flops[0];
  flops[1] = P->dev->launch_flops[1];
  return DMM_OK;
}

int dmm_plan_last_execute(const dmm_plan_t *P, dmm_execute_report *out) {
  if (!out) return DMM_EINVAL;
  *out = dmm_execute_report{0, 0, 0, 0};
  if (!P || !P->dev) return DMM_OK;
  out->ran_merged = P->dev->ran_merged ? 1 : 0;
  out->ran_k_split = P->dev->ran_k_split ? 1 : 0;
  out->ran_fused = P->dev->ran_fused;
  out->table_reused = P->dev->table_reused ? 1 : 0;
  return DMM_OK;
}

int dmm_plan_elapsed_ms(dmm_plan_t *P, float *gemm_ms, float *reduce_ms) {
  using namespace dmm;
  if (!P) return DMM_EINVAL;
  float g = -1.f, r = -1.f;
  if (P->dev && P->dev->gemm_timed) {
    DMM_HIP(hipEventSynchronize(P->dev->t_gemm[1]));
    DMM_HIP(hipEventElapsedTime(&g, P->dev->t_gemm[0], P->dev->t_gemm[1]));
  }
  if (P->dev && P->dev->red_timed) {
    DMM_HIP(hipEventSynchronize(P->dev->t_red[1]));
    DMM_HIP(hipEventElapsedTime(&r, P->dev->t_red[0], P->dev->t_red[1]));
  }
  if (gemm_ms) *gemm_ms = g;
  if (reduce_ms) *reduce_ms = r;
  return DMM_OK;
}

int dmm_reduce_replicas(dmm_plan_t *P, void *const *c_tiles, const int64_t *c_ld, int32_t origin_replica,
                        void *hip_stream) {
  using namespace dmm;
  if (!P || !c_tiles || !c_ld) return DMM_EINVAL;
  if (origin_replica < 0 || origin_replica >= P->C.c) return DMM_EINVAL;
  int rc;
  if ((rc = check_lds(P->C, c_ld))) return rc;
  TraceRange whole("dmm_reduce_replicas");
  try {
    if ((rc = ensure_state(P))) return rc;
    RedLaunch red;
    if ((rc = stage_reduce(P, c_tiles, c_ld, origin_replica, (hipStream_t)hip_stream, &red))) return rc;
    if ((rc = fire_reduce(P, red, (hipStream_t)hip_stream, false))) return rc;
    return P->C.c > 1 ? mark_use(P, (hipStream_t)hip_stream) : DMM_OK;
  } catch (const std::bad_alloc &) {
    return DMM_ENOMEM;
  }
}

int dmm_broadcast_replica(dmm_plan_t *P, void *const *c_tiles, const int64_t *c_ld, int32_t origin_replica,
                          void *hip_stream) {
  using namespace dmm;
  if (!P || !c_tiles || !c_ld) return DMM_EINVAL;
  if (origin_replica < 0 || origin_replica >= P->C.c) return DMM_EINVAL;
  int rc;
  if ((rc = check_lds(P->C, c_ld))) return rc;
  TraceRange whole("dmm_broadcast_replica");
  try {
    if ((rc = ensure_state(P))) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;
    RedLaunch L;
    if ((rc = stage_reduce(P, c_tiles, c_ld, origin_replica, stream, &L))) return rc;
    if (L.n_items == 0) return DMM_OK;
    char *d = L.dev_base;
    hipLaunchKernelGGL(broadcast_replica_kernel, dim3((unsigned)L.n_items), dim3(RED_NT), 0, stream,
                       (const RedItem *)(d + L.o_items), (const RedTile *)(d + L.o_tiles),
                       (float *const *)(d + L.o_parts), (const int64_t *)(d + L.o_lds), L.nparts, L.vec_ok ? 1 : 0);
    DMM_HIP(hipGetLastError());
    return mark_use(P, stream);
  } catch (const std::bad_alloc &) {
    return DMM_ENOMEM;
  }
}

}  // extern "C"

// ------------------------------------------------------------------ no allocation: static tables

// The replica sum's work tables for dmm_reduce_replicas_static.  In host code this name stands in
// for the symbol only: the memory is reached through the address hipGetSymbolAddress returns on
// each device (static_scratch below), never through the name.
static __device__ __align__(256) unsigned char scratch[DMM_STATIC_SCRATCH_BYTES];

namespace dmm {
namespace {

// Device address of `scratch` on the current device (every GPU holds its own copy), looked up
// once per device.
int static_scratch(char **out) {
  static std::mutex mu;
  static char *ptr[64] = {};
  int dev = 0;
  DMM_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return DMM_EINVAL;
  std::lock_guard<std::mutex> g(mu);
  if (!ptr[dev]) {
    void *p = nullptr;
    DMM_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return DMM_EHIP;
    ptr[dev] = (char *)p;
  }
  *out = ptr[dev];
  return DMM_OK;
}

// The tables of build_reduce, laid out the same way (items | tiles | part pointers | part lds),
// written into `dst` (capacity `cap` bytes) without any allocation: sizes first, then the records.
int build_reduce_in_place(const dmm_plan_t *P, void *const *c_tiles, const int64_t *c_ld, int32_t origin, char *dst,
                          size_t cap, RedLaunch *L, size_t *bytes) {
  const Grid &C = P->C;
  L->n_items = 0;
  *bytes = 0;
  if (C.c <= 1) return DMM_OK;
  const int nparts = C.c;
  auto rows_per_item = [](int64_t cols) { int64_t per = (RED_ELEMS + cols - 1) / cols; return per < 1 ? (int64_t)1 : per; };
  size_t n_tiles = 0, n_items = 0;
  for (int32_t ti = 0; ti < C.gr; ++ti)
    for (int32_t tj = 0; tj < C.gc; ++tj) {
      const int64_t rows = C.rc[ti + 1] - C.rc[ti], cols = C.cc[tj + 1] - C.cc[tj];
      if (rows <= 0 || cols <= 0) continue;
      const int64_t per = rows_per_item(cols);
      ++n_tiles;
      n_items += (size_t)((rows + per - 1) / per);
    }
  if (n_items == 0) return DMM_OK;
  const size_t o_items = 0;
  const size_t o_tiles = o_items + n_items * sizeof(RedItem);
  const size_t o_parts = o_tiles + n_tiles * sizeof(RedTile);
  const size_t o_lds = o_parts + n_tiles * (size_t)nparts * sizeof(void *);
  const size_t total = o_lds + n_tiles * (size_t)nparts * sizeof(int64_t);
  if (total > cap) return DMM_ELIMIT;
  RedItem *items = (RedItem *)(dst + o_items);
  RedTile *tiles = (RedTile *)(dst + o_tiles);
  const float **parts = (const float **)(dst + o_parts);
  int64_t *part_ld = (int64_t *)(dst + o_lds);
  bool vec_ok = true;
  size_t t_idx = 0, i_idx = 0;
  for (int32_t ti = 0; ti < C.gr; ++ti)
    for (int32_t tj = 0; tj < C.gc; ++tj) {
      const int64_t rows = C.rc[ti + 1] - C.rc[ti], cols = C.cc[tj + 1] - C.cc[tj];
      if (rows <= 0 || cols <= 0) continue;
      RedTile t;
      const int64_t oi = C.table_index(origin, ti, tj);
      t.out = (float *)c_tiles[oi];
      t.ldo = c_ld[oi];
      t.part_begin = (int64_t)(t_idx * (size_t)nparts);
      t.rows = (int32_t)rows;
      t.cols = (int32_t)cols;
      if (!t.out) return DMM_EINVAL;
      if (((uintptr_t)t.out & 15) || (t.ldo & 3) || (cols & 3)) vec_ok = false;
      for (int32_t rep = 0; rep < nparts; ++rep) {
        const int64_t pi = C.table_index(rep, ti, tj);
        const float *pp = (const float *)c_tiles[pi];
        if (!pp) return DMM_EINVAL;
        if (((uintptr_t)pp & 15) || (c_ld[pi] & 3)) vec_ok = false;
        parts[t_idx * (size_t)nparts + (size_t)rep] = pp;
        part_ld[t_idx * (size_t)nparts + (size_t)rep] = c_ld[pi];
      }
      const int64_t per = rows_per_item(cols);
      for (int64_t r = 0; r < rows; r += per) {
        RedItem it;
        it.tile = (int32_t)t_idx;
        it.row0 = (int32_t)r;
        it.nrows = (int32_t)(rows - r < per ? rows - r : per);
        it.pad = 0;
        items[i_idx++] = it;
      }
      tiles[t_idx++] = t;
    }
  L->n_items = n_items;
  L->o_items = o_items;
  L->o_tiles = o_tiles;
  L->o_parts = o_parts;
  L->o_lds = o_lds;
  L->nparts = nparts;
  L->vec_ok = vec_ok;
  *bytes = total;
  return DMM_OK;
}

}  // namespace
}  // namespace dmm

extern "C" int dmm_reduce_replicas_static(dmm_plan_t *P, void *const *c_tiles, const int64_t *c_ld,
                                          int32_t origin_replica, void *hip_stream) {
  using namespace dmm;
  if (!P || !c_tiles || !c_ld) return DMM_EINVAL;
  if (origin_replica < 0 || origin_replica >= P->C.c) return DMM_EINVAL;
  int rc;
  if ((rc = check_lds(P->C, c_ld))) return rc;
  hipStream_t stream = (hipStream_t)hip_stream;
  char *dev = nullptr;
  if ((rc = static_scratch(&dev))) return rc;
  // Fixed host buffers for all callers, taken in turn, one for the length of a call.  The copy
  // below reads pageable memory out (or stages it) before hipMemcpyAsync returns; taking four
  // buffers in turn means that even a copy that lagged behind its call would have to lag by four
  // calls to find its source overwritten.
  static std::mutex mu;
  constexpr int SLOTS = 4;
  alignas(16) static char slots[SLOTS][DMM_STATIC_SCRATCH_BYTES];
  static int next_slot = 0;
  std::lock_guard<std::mutex> g(mu);
  char *staging = slots[next_slot];
  RedLaunch L;
  size_t bytes = 0;
  if ((rc = build_reduce_in_place(P, c_tiles, c_ld, origin_replica, staging, DMM_STATIC_SCRATCH_BYTES, &L, &bytes))) return rc;
  if (L.n_items == 0) return DMM_OK;
  next_slot = (next_slot + 1) % SLOTS;
  DMM_HIP(hipMemcpyAsync(dev, staging, bytes, hipMemcpyHostToDevice, stream));
  hipLaunchKernelGGL(reduce_replicas_kernel, dim3((unsigned)L.n_items), dim3(RED_NT), 0, stream,
                     (const RedItem *)(dev + L.o_items), (const RedTile *)(dev + L.o_tiles),
                     (const float *const *)(dev + L.o_parts), (const int64_t *)(dev + L.o_lds), L.nparts, L.vec_ok ? 1 : 0);
  DMM_HIP(hipGetLastError());
  return DMM_OK;
}
