// Mapping of workgroup ids to work items that is aware of the chip's eight XCDs.
// The hardware hands workgroup b to XCD b % 8, in increasing b.  Work comes as `units`
// (a batch element x a kv head or head group: items of one unit read the same K/V or the
// same query tiles, so they should share an XCD's L2) of `per_unit` items each, ranked by
// decreasing work.  The map gives every XCD few units, the same amount of work (a unit's
// ranked items are dealt round-robin to the XCDs that share it), and starts the longest
// items first.
#pragma once
#include <stdint.h>

namespace loong {

struct WorkMap {
  int32_t units, per_unit;
  int32_t mode;   // 0: each XCD owns k whole units; 1: k XCDs share one unit; 2: plain round-robin
  int32_t k;
  uint32_t grid;  // workgroups to launch (a multiple of 8)
};

inline WorkMap make_work_map(int64_t units, int64_t per_unit) {
  WorkMap m{};
  m.units = (int32_t)units; m.per_unit = (int32_t)per_unit;
  if (units % 8 == 0) {
    m.mode = 0; m.k = (int32_t)(units / 8);
    m.grid = (uint32_t)(8 * m.k * per_unit);
  } else if (units < 8 && 8 % units == 0) {
    m.mode = 1; m.k = (int32_t)(8 / units);
    m.grid = (uint32_t)(8 * ((per_unit + m.k - 1) / m.k));
  } else {
    m.mode = 2; m.k = 1;
    m.grid = (uint32_t)((units * per_unit + 7) / 8 * 8);
  }
  return m;
}

// Work item of workgroup `block`: false if the workgroup is padding.
__device__ __forceinline__ bool decode_work(const WorkMap& m, uint32_t block, int& unit, int& rank) {
  const int xcd = block & 7, idx = block >> 3;
  if (m.mode == 0) {
    unit = xcd * m.k + idx % m.k;
    rank = idx / m.k;
  } else if (m.mode == 1) {
    unit = xcd / m.k;
    rank = idx * m.k + xcd % m.k;
  } else {
    rank = (int)(block / (uint32_t)m.units);
    unit = (int)(block % (uint32_t)m.units);
  }
  return rank < m.per_unit;
}

}  // namespace loong
