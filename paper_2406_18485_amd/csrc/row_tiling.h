// Host-side choice of the work split for the kernels whose workgroups own query rows
// (the forward step and the dQ pass of the backward step).  A workgroup has eight waves =
// NRB row blocks of 32 rows x KS key splits; GS heads of one kv group share a workgroup.
#pragma once
#include <cstdlib>

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

// number of q tiles of height bmh (rows per head) that have visible keys
inline int64_t busy_row_tiles(const StepGeom& g, int bmh) {
  int64_t n = 0;
  for (int a = 0; a < g.nq; ++a) {
    bool sees = false;
    for (int kb = 0; kb < g.nk; ++kb) sees |= g.cls[a][kb] != LOONG_SKIP && g.k[kb].len > 0;
    if (sees) n += (g.q[a].len + bmh - 1) / bmh;
  }
  return n;
}

// Key splits: more splits give more workgroups (each streams the whole visible K/V of its
// head through its own LDS), so splitting pays only while the chip is under-filled.  When
// one head's K/V chunk fits an XCD's L2 the aim is a workgroup on (nearly) every CU; when
// it does not, the extra streams cost more than the idle CUs and half the CUs is enough.
// The environment variable named by `env` (value 1, 2 or 4) overrides the choice (tuning aid).
inline int pick_key_splits(const StepGeom& g, int G, int Hq, int B, int head_dim, const char* env) {
  if (const char* e = std::getenv(env)) {
    const int v = std::atoi(e);
    if (v == 1 || v == 2 || v == 4) return v;
  }
  int64_t keys = 0;
  for (int kb = 0; kb < g.nk; ++kb) keys += g.k[kb].len;
  const int64_t kv_bytes = keys * head_dim * 2 * 2;
  const int64_t want = kv_bytes <= (3 << 20) ? 224 : 112;
  const int ks_opts[3] = {1, 2, 4};
  for (int i = 0; i < 3; ++i) {
    const int nrb = kRowWaves / ks_opts[i], gs = pick_gs(G, nrb);
    const int64_t n = busy_row_tiles(g, 32 * nrb / gs) * (Hq / gs) * B;
    if (n >= want) return ks_opts[i];
  }
  return 4;
}

// Placement of the row tiles of a launch with NRB row blocks per workgroup.
struct RowTiling {
  int GS, ntile[2], tiles_total, hgroups;
  int64_t total_wg;
};

inline RowTiling make_row_tiling(const StepGeom& g, int G, int Hq, int B, int nrb) {
  RowTiling t{};
  t.GS = pick_gs(G, nrb);
  const int bmh = 32 * nrb / t.GS;
  for (int a = 0; a < 2; ++a) {
    t.ntile[a] = a < g.nq ? (g.q[a].len + bmh - 1) / bmh : 0;
    t.tiles_total += t.ntile[a];
  }
  t.hgroups = Hq / t.GS;
  t.total_wg = (int64_t)t.tiles_total * t.hgroups * B;
  return t;
}

}  // namespace loong
