// Host-side choice of the work split for the kernels whose workgroups own query rows
// (the forward step and the dQ pass of the backward step).  A workgroup has eight waves =
// NRB row blocks of 32 rows x KS key splits; GS heads of one kv group share a workgroup.
#pragma once
#include "loong_internal.h"

namespace loong {

constexpr int kRowWaves = 8;

// heads of one kv group stacked in a workgroup: the largest power of two that divides the
// group size and fits the row blocks
inline int pick_gs(int G, int nrb) {
  for (int gs = 8; gs >= 1; gs >>= 1)
    if (G % gs == 0 && gs <= nrb) return gs;
  return 1;
}

// does q segment a see any key in this step?
inline bool segment_sees_keys(const StepGeom& g, int a) {
  for (int kb = 0; kb < g.nk; ++kb)
    if (g.cls[a][kb] != LOONG_SKIP && g.k[kb].len > 0) return true;
  return false;
}

// number of q tiles of height bmh (rows per head) that have visible keys
inline int64_t busy_row_tiles(const StepGeom& g, int bmh) {
  int64_t n = 0;
  for (int a = 0; a < g.nq; ++a)
    if (segment_sees_keys(g, a)) n += (g.q[a].len + bmh - 1) / bmh;
  return n;
}

// Key splits: more splits give more workgroups, but each workgroup streams the whole visible
// K/V of its head through its own LDS and keeps fewer rows per staged tile, so the smallest
// split that puts a workgroup on (nearly) every compute unit is taken (measured on
// 32K..1M-token shapes: one more split than that is always slower, one fewer leaves units idle).
// `forced` (1, 2 or 4, from the descriptor's flags) overrides the choice; `cus` is the device's
// number of compute units.
inline int pick_key_splits(const StepGeom& g, int G, int Hq, int B, int forced, int cus) {
  if (forced == 1 || forced == 2 || forced == 4) return forced;
  // a step with a diagonal block has tiles of very different length: two workgroups per unit,
  // longest first, even them out
  bool diag = false;
  for (int a = 0; a < g.nq; ++a)
    for (int kb = 0; kb < g.nk; ++kb) diag |= g.cls[a][kb] == LOONG_DIAG;
  const int64_t want = (diag ? 2 : 1) * (int64_t)cus * 7 / 8;
  const int ks_opts[3] = {1, 2, 4};
  for (int i = 0; i < 3; ++i) {
    const int nrb = kRowWaves / ks_opts[i], gs = pick_gs(G, nrb);
    const int64_t n = busy_row_tiles(g, 32 * nrb / gs) * (Hq / gs) * B;
    if (n >= want) return ks_opts[i];
  }
  return 4;
}

// Placement of the row tiles of a launch with NRB row blocks per workgroup.  With
// `list_blind` false, q segments that see no key in this step get no tiles at all: the work
// list then holds busy tiles only, and cutting it into eight equal ranges (one per XCD)
// balances the chip.
struct RowTiling {
  int GS, ntile[2], tiles_total, hgroups;
  int64_t total_wg;
};

inline RowTiling make_row_tiling(const StepGeom& g, int G, int Hq, int B, int nrb, bool list_blind) {
  RowTiling t{};
  t.GS = pick_gs(G, nrb);
  const int bmh = 32 * nrb / t.GS;
  for (int a = 0; a < 2; ++a) {
    t.ntile[a] = a < g.nq && (list_blind || segment_sees_keys(g, a)) ? (g.q[a].len + bmh - 1) / bmh : 0;
    t.tiles_total += t.ntile[a];
  }
  t.hgroups = Hq / t.GS;
  t.total_wg = (int64_t)t.tiles_total * t.hgroups * B;
  return t;
}

}  // namespace loong
