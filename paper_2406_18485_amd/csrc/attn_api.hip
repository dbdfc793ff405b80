// C entry points of the forward and backward micro-step: validate, then dispatch on dtype.
#include <hip/hip_runtime.h>

#include "loong_internal.h"

using namespace loong;

extern "C" {

int loong_attn_step_fwd(const loong_step_desc* desc, const void* q, const void* k, const void* v,
                        float* out, float* lse, void* stream) {
  clear_error();
  StepGeom g;
  if (int rc = check_step(desc, &g)) return rc;
  if (!q || !k || !v || !out || !lse) return fail(LOONG_E_NULL, "loong_attn_step_fwd: NULL tensor");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out))
    return fail(LOONG_E_ALIGN, "loong_attn_step_fwd: q/k/v/out must be 16-byte aligned");
  if (desc->batch == 0 || desc->q_len == 0) return LOONG_OK;
  return desc->dtype == LOONG_FP32 ? launch_fwd_f32(*desc, g, q, k, v, out, lse, stream)
                                   : launch_fwd_bf16(*desc, g, q, k, v, out, lse, stream);
}

int loong_attn_step_bwd(const loong_step_desc* desc, const void* q, const void* k, const void* v,
                        const void* o, const void* d_o, const float* lse, float* delta, float* dq,
                        float* dk, float* dv, void* workspace, int64_t workspace_bytes, void* stream) {
  clear_error();
  StepGeom g;
  if (int rc = check_step(desc, &g)) return rc;
  const bool only_dkv = desc->flags & LOONG_BWD_ONLY_DKV, only_dq = desc->flags & LOONG_BWD_ONLY_DQ;
  if (only_dkv && only_dq)
    return fail(LOONG_E_UNSUPPORTED, "loong_attn_step_bwd: LOONG_BWD_ONLY_DKV and LOONG_BWD_ONLY_DQ exclude each other");
  if (!q || !k || !v || !d_o || !lse || !delta || (!only_dkv && !dq) || (!only_dq && (!dk || !dv)))
    return fail(LOONG_E_NULL, "loong_attn_step_bwd: NULL tensor");
  const bool want_delta = desc->flags & LOONG_COMPUTE_DELTA;
  if (want_delta && !o) return fail(LOONG_E_NULL, "loong_attn_step_bwd: LOONG_COMPUTE_DELTA needs o");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(d_o) || (!only_dkv && !aligned16(dq)) ||
      (!only_dq && (!aligned16(dk) || !aligned16(dv))) || (want_delta && !aligned16(o)))
    return fail(LOONG_E_ALIGN, "loong_attn_step_bwd: tensors must be 16-byte aligned");
  if (workspace_bytes < 0) return fail(LOONG_E_SHAPE, "loong_attn_step_bwd: negative workspace size");
  if (desc->batch == 0) return LOONG_OK;
  if (desc->dtype != LOONG_FP32) {  // scratch for shared query loops: checked before anything is enqueued
    const int64_t need = bwd_workspace_bytes_bf16(*desc, g);
    if (need > 0) {
      if (!workspace)
        return fail(LOONG_E_NULL, "loong_attn_step_bwd: this step needs a workspace of %lld bytes (loong_workspace_bytes)",
                    (long long)need);
      if (!aligned16(workspace)) return fail(LOONG_E_ALIGN, "loong_attn_step_bwd: the workspace must be 16-byte aligned");
      if (workspace_bytes < need)
        return fail(LOONG_E_SHAPE, "loong_attn_step_bwd: workspace of %lld bytes, this step needs %lld (loong_workspace_bytes)",
                    (long long)workspace_bytes, (long long)need);
    }
  }
  if (want_delta)
    if (int rc = loong_bwd_delta(desc, o, d_o, delta, stream)) return rc;
  return desc->dtype == LOONG_FP32
             ? launch_bwd_f32(*desc, g, q, k, v, d_o, lse, delta, dq, dk, dv, stream)
             : launch_bwd_bf16(*desc, g, q, k, v, d_o, lse, delta, dq, dk, dv, workspace, workspace_bytes, stream);
}

int loong_workspace_bytes(const loong_step_desc* desc, int64_t* bytes) {
  clear_error();
  StepGeom g;
  if (int rc = check_step(desc, &g)) return rc;
  if (!bytes) return fail(LOONG_E_NULL, "loong_workspace_bytes: NULL result");
  *bytes = desc->dtype == LOONG_FP32 ? 0 : bwd_workspace_bytes_bf16(*desc, g);
  return LOONG_OK;
}

}  // extern "C"
