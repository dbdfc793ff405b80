// Performance model of 2D-Attention (paper: Sec. "Performance Analysis"): closed forms for the
// compute time of a micro-step, the bytes of a K/V chunk, the overlapped time of an inner
// ring and the all-to-all traffic, and the search for the best (d_hp, d_cp, w).  Host only.
#include <algorithm>
#include <cmath>

#include "loong_internal.h"

namespace loong {
namespace {

int check_cost_in(const loong_cost_in* in, bool with_grid) {
  if (!in) return fail(LOONG_E_NULL, "cost model: input is NULL");
  if (!(in->S > 0) || !(in->D > 0) || in->H < 1 || in->H_kv < 1 || in->H % in->H_kv != 0)
    return fail(LOONG_E_SHAPE, "cost model: S, D, H, H_kv must be positive and H_kv must divide H");
  if (!(in->alpha_fwd > 0) || !(in->bw_p2p_inner > 0) || !(in->bw_p2p_outer > 0) || !(in->bw_alltoall > 0) ||
      !(in->latency >= 0))
    return fail(LOONG_E_SHAPE, "cost model: alpha and bandwidths must be positive, latency non-negative");
  if (with_grid) {
    if (in->d_hp < 1 || in->d_cp < 1 || in->w < 1)
      return fail(LOONG_E_SHAPE, "cost model: d_hp, d_cp, w must be positive");
    if (in->H % in->d_hp != 0) return fail(LOONG_E_SHAPE, "cost model: d_hp %d does not divide H %d", in->d_hp, in->H);
    if (in->d_cp % in->w != 0) return fail(LOONG_E_SHAPE, "cost model: w %d does not divide d_cp %d", in->w, in->d_cp);
  }
  return LOONG_OK;
}

void evaluate(const loong_cost_in& in, loong_cost_out& o) {
  const double d_sp = (double)in.d_hp * in.d_cp;
  // Size(kv): K and V of the (possibly replicated) local heads, 16-bit elements
  o.size_kv = (double)std::max(in.H_kv, in.d_hp) / in.H * 4.0 * in.S * in.D / d_sp;
  o.size_q = 2.0 * in.S * in.D / d_sp;
  o.alltoall_volume = (2.0 * o.size_q + o.size_kv) * (in.d_hp - 1) / in.d_hp;
  o.t_comp_fwd = in.alpha_fwd * in.S * in.S * in.D / (in.d_cp * d_sp);
  o.t_comp_bwd = 3.0 * o.t_comp_fwd;
  o.t_p2p_inner_fwd = in.latency + o.size_kv / in.bw_p2p_inner;
  o.t_p2p_outer_fwd = in.latency + o.size_kv / in.bw_p2p_outer;
  o.t_p2p_inner_bwd = in.latency + 2.0 * o.size_kv / in.bw_p2p_inner;  // chunk + its gradient
  o.t_p2p_outer_bwd = in.latency + 2.0 * o.size_kv / in.bw_p2p_outer;
  o.t_inner_ring_fwd = std::max(o.t_comp_fwd, o.t_p2p_inner_fwd) * (in.w - 1) + std::max(o.t_comp_fwd, o.t_p2p_outer_fwd);
  o.t_inner_ring_bwd = std::max(o.t_comp_bwd, o.t_p2p_inner_bwd) * (in.w - 1) + std::max(o.t_comp_bwd, o.t_p2p_outer_bwd);
  o.t_seq_alltoall = in.d_hp > 1 ? 2.0 * o.alltoall_volume / in.bw_alltoall : 0.0;
  o.objective = o.t_seq_alltoall + (o.t_inner_ring_fwd + o.t_inner_ring_bwd) * ((double)in.d_cp / in.w);
}

}  // namespace
}  // namespace loong

extern "C" {

int loong_cost_model(const loong_cost_in* in, loong_cost_out* out) {
  loong::clear_error();
  if (int rc = loong::check_cost_in(in, true)) return rc;
  if (!out) return loong::fail(LOONG_E_NULL, "cost model: output is NULL");
  loong::evaluate(*in, *out);
  return LOONG_OK;
}

int loong_cost_search(const loong_cost_in* in, int32_t d_sp, int32_t max_w, loong_cost_in* best_in,
                      loong_cost_out* best_out) {
  loong::clear_error();
  if (int rc = loong::check_cost_in(in, false)) return rc;
  if (!best_in || !best_out) return loong::fail(LOONG_E_NULL, "cost search: output is NULL");
  if (d_sp < 1 || max_w < 1) return loong::fail(LOONG_E_SHAPE, "cost search: d_sp and max_w must be positive");
  bool found = false;
  for (int32_t hp = 1; hp <= d_sp && hp <= in->H; ++hp) {
    if (d_sp % hp != 0 || in->H % hp != 0) continue;
    const int32_t cp = d_sp / hp;
    for (int32_t w = 1; w <= max_w && w <= cp; ++w) {
      if (cp % w != 0) continue;
      loong_cost_in cand = *in;
      cand.d_hp = hp; cand.d_cp = cp; cand.w = w;
      loong_cost_out o;
      loong::evaluate(cand, o);
      if (!found || o.objective < best_out->objective) {
        *best_in = cand;
        *best_out = o;
        found = true;
      }
    }
  }
  if (!found) return loong::fail(LOONG_E_SHAPE, "cost search: no admissible grid for d_sp %d", d_sp);
  return LOONG_OK;
}

}  // extern "C"
