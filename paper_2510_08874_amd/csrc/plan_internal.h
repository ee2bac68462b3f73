// Internal layout of a plan, shared by the host planner (plan.cpp) and the
// executor (exec.hip).  Not part of the ABI.
#pragma once

#include <cstdint>
#include <vector>

#include "dmm.h"

namespace dmm {

constexpr int32_t kMacroTile = 256;  // edge of the square C macro-tile one workgroup owns

struct Grid {                         // one distributed matrix (Section 3)
  int64_t rows = 0, cols = 0;
  std::vector<int64_t> rc, cc;        // cut points per axis
  int32_t gr = 0, gc = 0;             // tile grid
  int32_t pr = 1, pc = 1;             // process grid inside a replica
  int32_t c = 1;                      // replication factor
  int64_t tiles_per_rep() const { return (int64_t)gr * gc; }
  int64_t table_index(int32_t rep, int32_t ti, int32_t tj) const {
    return rep * tiles_per_rep() + (int64_t)ti * gc + tj;
  }
};

struct Group {                        // one output sub-tile and its K-segments
  int64_t m0, m1, n0, n1;
  int32_t c_rep, c_ti, c_tj;
  int64_t first, count;               // range in `order`
};

// Merged macro-tiles (Stationary C whose replicas each read one replica of A and of B): all ops
// of one C replica are the cells of one grid, (merged row cuts) x (K-segments of the replica's
// share) x (merged column cuts), so a macro-tile can be cut from the replica as a whole, across
// tile boundaries, and is described by the row intervals and column intervals it meets.
constexpr int32_t kMaxPieces = 8;     // row (column) intervals one merged macro-tile may meet
constexpr int32_t kPieceAlign = 8;    // column pieces start at multiples of this many columns inside the macro-tile
constexpr int64_t kDescBytes = 32 * 1024 - 2048;  // room for one macro-tile's descriptors on the device:
                                                   // 4 bytes per segment + 24 per (segment, piece)

struct MergedRep {
  std::vector<int64_t> kc;            // segment boundaries inside the replica's share of k
  int32_t a_rep = 0, b_rep = 0;       // the replicas of A and B this C replica's ranks read
};

struct MergedItem {
  int64_t m0, n0;
  int32_t m_ext, n_ext;
  int32_t rep;
  int32_t mr0, R, nr0, Q;             // first row interval, row pieces, first column interval, column pieces
};

constexpr int32_t kSegWindow = 64;    // segments a macro-tile is run on at a time where all of them would crowd
                                      // out the pieces (see Merged::window)
constexpr int32_t kMinPieces = 6;     // ... which is when fewer than this many pieces per axis would fit

struct Merged {
  bool valid = false;
  // 0: a macro-tile's workgroup walks all K-segments of its replica.  Otherwise the descriptors of
  // all segments would leave room for fewer than kMinPieces pieces per axis, and the executor runs
  // every macro-tile in windows of at most this many segments, whose partial tiles it adds up.
  int32_t window = 0;
  std::vector<int64_t> mc, nc;        // merged row cuts of A and C, merged column cuts of B and C
  std::vector<MergedRep> reps;
  std::vector<MergedItem> items;      // launch order
  std::vector<dmm_merged_item> view;  // the same list as the ABI shows it
};

struct DeviceState;                   // owned by exec.hip

}  // namespace dmm

struct dmm_plan_s {
  dmm::Grid A, B, C;
  int32_t nranks = 0;
  uint32_t flags = 0;                 // of dmm_plan
  bool listed = false;                // tasks, order, groups and items have been written out
  std::vector<dmm_task> tasks;        // Algorithm-1 order
  std::vector<int64_t> order;         // grouped order
  std::vector<int64_t> group_offsets; // groups + 1
  std::vector<dmm::Group> groups;
  std::vector<dmm_work_item> items;   // launch order
  dmm::Merged merged;                 // the alternative to `items` where it pays
  dmm::DeviceState *dev = nullptr;
};

namespace dmm {
void destroy_device_state(DeviceState *);  // exec.hip
// Writes out the op list, its grouped order and the per-group macro-tiles if that has not happened
// yet (a plan with a merged work list leaves them until somebody needs them).  DMM_OK or DMM_ENOMEM.
int materialize(dmm_plan_t *P);            // plan.cpp
}
