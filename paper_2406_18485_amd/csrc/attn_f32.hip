// fp32-storage kernels of the ring step (small cases, e.g. the fp32 tiny benchmark shape).
// One wave per row, plain fp32 FMAs, no matrix cores: written for clarity and a fixed
// order of operations, not for speed.  The bf16 MFMA kernels are the tuned path.
#include <hip/hip_runtime.h>

#include "device_utils.h"
#include "loong_internal.h"

namespace loong {
namespace {

struct F32Params {
  const float *q, *k, *v, *d_o, *lse_in, *delta;
  float *out, *lse, *dq, *dk, *dv;
  int B, Hq, Hkv, G, d, q_len, kv_len;
  int64_t qs[3], ks[3], os[3];
  StepGeom g;
  float scale;
  int flags;
};

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) x = fmaxf(x, __shfl_xor(x, m, 64));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) x += __shfl_xor(x, m, 64);
  return x;
}

// dot product of an LDS-resident row with a global row, d a multiple of 4
__device__ __forceinline__ float dot_row(const float* __restrict__ a_lds, const float* __restrict__ g, int d) {
  float s = 0.f;
  for (int t = 0; t < d; t += 4) {
    const float4 x = *reinterpret_cast<const float4*>(g + t);
    s += a_lds[t] * x.x + a_lds[t + 1] * x.y + a_lds[t + 2] * x.z + a_lds[t + 3] * x.w;
  }
  return s;
}

// Number of leading keys of key segment kb visible to the row at offset qoff of q segment qa.
__device__ __forceinline__ int visible_keys(const StepGeom& g, int qa, int kb, int qoff) {
  const int cls = g.cls[qa][kb];
  if (cls == LOONG_SKIP) return 0;
  const int len = g.k[kb].len;
  return cls == LOONG_FULL ? len : min(len, qoff + 1);
}

// ---- forward: one wave per query row --------------------------------------------------
__global__ __launch_bounds__(64) void fwd_f32_kernel(F32Params p) {
  __shared__ float q_s[128];
  const int lane = threadIdx.x;
  const int64_t rid = blockIdx.x;
  const int i = (int)(rid % p.q_len);
  const int h = (int)((rid / p.q_len) % p.Hq);
  const int64_t b = rid / ((int64_t)p.q_len * p.Hq);
  const int hk = h / p.G;
  const float* qrow = p.q + b * p.qs[0] + h * p.qs[1] + (int64_t)i * p.qs[2];
  for (int t = lane; t < p.d; t += 64) q_s[t] = qrow[t];
  __syncthreads();
  const int qa = (p.g.nq == 2 && i >= p.g.q[1].start) ? 1 : 0;
  const int qoff = i - p.g.q[qa].start;
  const bool fuse = p.flags & LOONG_FUSE_MERGE;
  float* orow = p.out + b * p.os[0] + h * p.os[1] + (int64_t)i * p.os[2];
  float* lse_p = p.lse + (b * p.Hq + h) * (int64_t)p.q_len + i;

  float m = -INFINITY, l = 0.f, acc0 = 0.f, acc1 = 0.f;
  if (fuse) {
    const float prev = *lse_p;
    if (prev != -INFINITY) {
      m = prev * kLog2e;
      l = 1.f;
      if (lane < p.d) acc0 = orow[lane];
      if (lane + 64 < p.d) acc1 = orow[lane + 64];
    }
  }
  bool any_key = false;
  const float c = p.scale * kLog2e;
  for (int kb = 0; kb < p.g.nk; ++kb) {
    const int kmax = visible_keys(p.g, qa, kb, qoff);
    const float* kbase = p.k + b * p.ks[0] + hk * p.ks[1] + (int64_t)p.g.k[kb].start * p.ks[2];
    const float* vbase = p.v + b * p.ks[0] + hk * p.ks[1] + (int64_t)p.g.k[kb].start * p.ks[2];
    for (int j0 = 0; j0 < kmax; j0 += 64) {
      any_key = true;
      const int j = j0 + lane;
      const bool valid = j < kmax;
      float s = dot_row(q_s, kbase + (int64_t)min(j, kmax - 1) * p.ks[2], p.d) * c;
      s = valid ? s : -INFINITY;
      const float m_new = fmaxf(m, wave_max(s));  // finite: lane 0 is always valid
      const float alpha = fast_exp2(m - m_new);   // m = -inf gives 0
      const float pj = fast_exp2(s - m_new);
      l = l * alpha + wave_sum(pj);
      acc0 *= alpha;
      acc1 *= alpha;
      const int cnt = min(64, kmax - j0);
      for (int t = 0; t < cnt; ++t) {
        const float pt = __shfl(pj, t, 64);
        const float* vrow = vbase + (int64_t)(j0 + t) * p.ks[2];
        if (lane < p.d) acc0 += pt * vrow[lane];
        if (lane + 64 < p.d) acc1 += pt * vrow[lane + 64];
      }
      m = m_new;
    }
  }
  if (!any_key) {
    if (fuse) return;  // running result untouched
    if (lane < p.d) orow[lane] = 0.f;
    if (lane + 64 < p.d) orow[lane + 64] = 0.f;
    if (lane == 0) *lse_p = -INFINITY;
    return;
  }
  const float inv = 1.f / l;
  if (lane < p.d) orow[lane] = acc0 * inv;
  if (lane + 64 < p.d) orow[lane + 64] = acc1 * inv;
  if (lane == 0) *lse_p = (m + fast_log2(l)) * kLn2;
}

// ---- backward, dQ share: one wave per query row -----------------------------------------
__global__ __launch_bounds__(64) void bwd_dq_f32_kernel(F32Params p) {
  __shared__ float q_s[128], do_s[128];
  const int lane = threadIdx.x;
  const int64_t rid = blockIdx.x;
  const int i = (int)(rid % p.q_len);
  const int h = (int)((rid / p.q_len) % p.Hq);
  const int64_t b = rid / ((int64_t)p.q_len * p.Hq);
  const int hk = h / p.G;
  const int64_t qoffs = b * p.qs[0] + h * p.qs[1] + (int64_t)i * p.qs[2];
  for (int t = lane; t < p.d; t += 64) {
    q_s[t] = p.q[qoffs + t];
    do_s[t] = p.d_o[qoffs + t];
  }
  __syncthreads();
  const int64_t srow = (b * p.Hq + h) * (int64_t)p.q_len + i;
  const float lse_i = p.lse_in[srow], dl = p.delta[srow];
  if (lse_i == -INFINITY) return;
  const int qa = (p.g.nq == 2 && i >= p.g.q[1].start) ? 1 : 0;
  const int qoff = i - p.g.q[qa].start;
  float acc0 = 0.f, acc1 = 0.f;
  for (int kb = 0; kb < p.g.nk; ++kb) {
    const int kmax = visible_keys(p.g, qa, kb, qoff);
    const float* kbase = p.k + b * p.ks[0] + hk * p.ks[1] + (int64_t)p.g.k[kb].start * p.ks[2];
    const float* vbase = p.v + b * p.ks[0] + hk * p.ks[1] + (int64_t)p.g.k[kb].start * p.ks[2];
    for (int j0 = 0; j0 < kmax; j0 += 64) {
      const int j = j0 + lane;
      const bool valid = j < kmax;
      const int64_t off = (int64_t)min(j, kmax - 1) * p.ks[2];
      const float s = dot_row(q_s, kbase + off, p.d) * p.scale;
      const float pj = valid ? fast_exp2((s - lse_i) * kLog2e) : 0.f;
      const float dp = dot_row(do_s, vbase + off, p.d);
      const float ds = pj * (dp - dl) * p.scale;
      const int cnt = min(64, kmax - j0);
      for (int t = 0; t < cnt; ++t) {
        const float dst = __shfl(ds, t, 64);
        const float* krow = kbase + (int64_t)(j0 + t) * p.ks[2];
        if (lane < p.d) acc0 += dst * krow[lane];
        if (lane + 64 < p.d) acc1 += dst * krow[lane + 64];
      }
    }
  }
  float* dqrow = p.dq + b * p.os[0] + h * p.os[1] + (int64_t)i * p.os[2];
  if (lane < p.d) dqrow[lane] += acc0;
  if (lane + 64 < p.d) dqrow[lane + 64] += acc1;
}

// ---- backward, dK/dV of the visiting chunk: one wave per key row ---------------------------
__global__ __launch_bounds__(64) void bwd_dkv_f32_kernel(F32Params p) {
  __shared__ float k_s[128], v_s[128];
  const int lane = threadIdx.x;
  const int64_t rid = blockIdx.x;
  const int j = (int)(rid % p.kv_len);
  const int hk = (int)((rid / p.kv_len) % p.Hkv);
  const int64_t b = rid / ((int64_t)p.kv_len * p.Hkv);
  const int64_t koffs = b * p.ks[0] + hk * p.ks[1] + (int64_t)j * p.ks[2];
  for (int t = lane; t < p.d; t += 64) {
    k_s[t] = p.k[koffs + t];
    v_s[t] = p.v[koffs + t];
  }
  __syncthreads();
  const int kb = (p.g.nk == 2 && j >= p.g.k[1].start) ? 1 : 0;
  const int koff = j - p.g.k[kb].start;
  float ak0 = 0.f, ak1 = 0.f, av0 = 0.f, av1 = 0.f;
  for (int gq = 0; gq < p.G; ++gq) {
    const int h = hk * p.G + gq;
    for (int qa = 0; qa < p.g.nq; ++qa) {
      const int cls = p.g.cls[qa][kb];
      if (cls == LOONG_SKIP) continue;
      const int len = p.g.q[qa].len;
      const int first = cls == LOONG_DIAG ? koff : 0;  // rows at or after the key see it
      const int64_t qbase = b * p.qs[0] + h * p.qs[1] + (int64_t)p.g.q[qa].start * p.qs[2];
      const int64_t sbase = (b * p.Hq + h) * (int64_t)p.q_len + p.g.q[qa].start;
      for (int i0 = first; i0 < len; i0 += 64) {
        const int i = i0 + lane;
        const bool valid = i < len;
        const int ic = min(i, len - 1);
        const float lse_i = p.lse_in[sbase + ic], dl = p.delta[sbase + ic];
        const float s = dot_row(k_s, p.q + qbase + (int64_t)ic * p.qs[2], p.d) * p.scale;
        const float pi = (valid && lse_i != -INFINITY) ? fast_exp2((s - lse_i) * kLog2e) : 0.f;
        const float dp = dot_row(v_s, p.d_o + qbase + (int64_t)ic * p.qs[2], p.d);
        const float ds = pi * (dp - dl) * p.scale;
        const int cnt = min(64, len - i0);
        for (int t = 0; t < cnt; ++t) {
          const float pt = __shfl(pi, t, 64), dst = __shfl(ds, t, 64);
          const float* qrow = p.q + qbase + (int64_t)(i0 + t) * p.qs[2];
          const float* dorow = p.d_o + qbase + (int64_t)(i0 + t) * p.qs[2];
          if (lane < p.d) {
            ak0 += dst * qrow[lane];
            av0 += pt * dorow[lane];
          }
          if (lane + 64 < p.d) {
            ak1 += dst * qrow[lane + 64];
            av1 += pt * dorow[lane + 64];
          }
        }
      }
    }
  }
  const int64_t orow = ((b * p.Hkv + hk) * (int64_t)p.kv_len + j) * p.d;
  const bool accum = p.flags & LOONG_ACCUM_DKV;
  if (lane < p.d) {
    p.dk[orow + lane] = (accum ? p.dk[orow + lane] : 0.f) + ak0;
    p.dv[orow + lane] = (accum ? p.dv[orow + lane] : 0.f) + av0;
  }
  if (lane + 64 < p.d) {
    p.dk[orow + lane + 64] = (accum ? p.dk[orow + lane + 64] : 0.f) + ak1;
    p.dv[orow + lane + 64] = (accum ? p.dv[orow + lane + 64] : 0.f) + av1;
  }
}

F32Params make_params(const loong_step_desc& d, const StepGeom& g) {
  F32Params p{};
  p.B = d.batch; p.Hq = d.n_q_heads; p.Hkv = d.n_kv_heads; p.G = d.n_q_heads / d.n_kv_heads;
  p.d = d.head_dim; p.q_len = d.q_len; p.kv_len = d.kv_len;
  for (int i = 0; i < 3; ++i) { p.qs[i] = d.q_stride[i]; p.ks[i] = d.kv_stride[i]; p.os[i] = d.o_stride[i]; }
  p.g = g; p.scale = d.softmax_scale; p.flags = d.flags;
  return p;
}

}  // namespace

int launch_fwd_f32(const loong_step_desc& d, const StepGeom& g, const void* q, const void* k,
                   const void* v, float* out, float* lse, void* stream) {
  const int64_t rows = (int64_t)d.batch * d.n_q_heads * d.q_len;
  if (rows == 0) return LOONG_OK;
  if (rows > 0x7fffffff) return fail(LOONG_E_UNSUPPORTED, "fp32 path: more than 2^31-1 query rows");
  F32Params p = make_params(d, g);
  p.q = (const float*)q; p.k = (const float*)k; p.v = (const float*)v; p.out = out; p.lse = lse;
  fwd_f32_kernel<<<dim3((unsigned)rows), dim3(64), 0, static_cast<hipStream_t>(stream)>>>(p);
  return check_launch("loong_attn_step_fwd (fp32)");
}

int launch_bwd_f32(const loong_step_desc& d, const StepGeom& g, const void* q, const void* k,
                   const void* v, const void* d_o, const float* lse, const float* delta, float* dq,
                   float* dk, float* dv, void* stream) {
  const int64_t qrows = (int64_t)d.batch * d.n_q_heads * d.q_len;
  const int64_t krows = (int64_t)d.batch * d.n_kv_heads * d.kv_len;
  if (qrows > 0x7fffffff || krows > 0x7fffffff)
    return fail(LOONG_E_UNSUPPORTED, "fp32 path: more than 2^31-1 rows");
  F32Params p = make_params(d, g);
  p.q = (const float*)q; p.k = (const float*)k; p.v = (const float*)v; p.d_o = (const float*)d_o;
  p.lse_in = lse; p.delta = delta; p.dq = dq; p.dk = dk; p.dv = dv;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool do_dq = !(d.flags & LOONG_BWD_ONLY_DKV), do_dkv = !(d.flags & LOONG_BWD_ONLY_DQ);
  if (do_dq && qrows > 0 && krows > 0) {
    bwd_dq_f32_kernel<<<dim3((unsigned)qrows), dim3(64), 0, st>>>(p);
    if (int rc = check_launch("loong_attn_step_bwd (fp32 dq)")) return rc;
  }
  if (do_dkv && krows > 0) {
    bwd_dkv_f32_kernel<<<dim3((unsigned)krows), dim3(64), 0, st>>>(p);
    if (int rc = check_launch("loong_attn_step_bwd (fp32 dk/dv)")) return rc;
  }
  return LOONG_OK;
}

}  // namespace loong
