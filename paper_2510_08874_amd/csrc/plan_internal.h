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

struct DeviceState;                   // owned by exec.hip

}  // namespace dmm

struct dmm_plan_s {
  dmm::Grid A, B, C;
  int32_t nranks = 0;
  std::vector<dmm_task> tasks;        // Algorithm-1 order
  std::vector<int64_t> order;         // grouped order
  std::vector<int64_t> group_offsets; // groups + 1
  std::vector<dmm::Group> groups;
  std::vector<dmm_work_item> items;   // launch order
  dmm::DeviceState *dev = nullptr;
};

namespace dmm {
void destroy_device_state(DeviceState *);  // exec.hip
}
