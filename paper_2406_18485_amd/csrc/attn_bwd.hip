// Backward micro-step on bf16 matrix cores: gradients of the visiting K/V chunk and this
// step's share of dQ, recomputing the probabilities from the final softmax_lse
// (paper: Sec. 3.1 last paragraph; Sec. "Selective Checkpoint++").
//
// Work split.  A workgroup of 4 waves owns 128 keys of one kv head (32 per wave) and walks
// over the query tiles (64 rows) of every q head of the group that can see them.  The
// wave's K and V rows stay in registers as B operands of S = Q K^T and dP = dO V^T, whose
// accumulators put one key per lane and 16 query rows per 32x32 block in registers: that
// is the A-operand layout for dV += P^T dO and dK += dS^T Q (contraction over rows), with
// dO and Q read from LDS as row pairs interleaved per column.  dS goes through LDS once,
// transposed by the write, so that dQ = dS K contracts over all 128 keys; each wave adds
// one 32-column block of the dQ tile to global memory with fp32 atomics.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "device_utils.h"
#include "loong_internal.h"

namespace loong {
namespace {

struct BwdParams {
  const uint16_t *q, *k, *v, *d_o;
  const float *lse, *delta;
  float *dq, *dk, *dv;
  int B, Hq, Hkv, G;
  int q_len, kv_len;
  int64_t qs[3], ks[3], os[3];
  StepGeom g;
  float scale, c;  // softmax scale; scale * log2(e)
  int add_dkv;     // 1: dk/dv are added to with atomics (accumulate flag or split iteration space)
  int nkt[2], kt_total;
  int nsplit;
  int total_wg;
};

constexpr int kBwdWaves = 4;
constexpr int kBwdBN = 32 * kBwdWaves;

// interleave two rows' 8-column pieces into per-column (row0, row1) dwords
__device__ __forceinline__ void interleave_rows(const uint4 a, const uint4 b, uint4& w0, uint4& w1) {
  w0.x = (a.x & 0xffffu) | (b.x << 16); w0.y = (a.x >> 16) | (b.x & 0xffff0000u);
  w0.z = (a.y & 0xffffu) | (b.y << 16); w0.w = (a.y >> 16) | (b.y & 0xffff0000u);
  w1.x = (a.z & 0xffffu) | (b.z << 16); w1.y = (a.z >> 16) | (b.z & 0xffff0000u);
  w1.z = (a.w & 0xffffu) | (b.w << 16); w1.w = (a.w >> 16) | (b.w & 0xffff0000u);
}

template <int D, int BM>
__global__ __launch_bounds__(kBwdWaves * 64) void bwd_kernel(const BwdParams p) {
  constexpr int NT = kBwdWaves * 64, BN = kBwdBN;
  constexpr int NKS = D / 16, NDB = D / 32, NIB = BM / 32, CPR = D / 8;
  constexpr int RSTR = D + 8;    // bf16 per row of the row-major Q / dO tiles
  constexpr int PSTR = D + 16;   // dwords per row of the pair-interleaved tiles
  constexpr int SSTR = BN + 8;   // bf16 per row of the dS tile
  constexpr int T_UNITS = (BM / 2) * CPR, T_PT = (T_UNITS + NT - 1) / NT;
  constexpr int K_UNITS = (BN / 2) * CPR, K_PT = (K_UNITS + NT - 1) / NT;
  __shared__ __attribute__((aligned(16))) uint16_t Qs[BM * RSTR];
  __shared__ __attribute__((aligned(16))) uint16_t dOs[BM * RSTR];
  __shared__ __attribute__((aligned(16))) uint32_t Qp[(BM / 2) * PSTR];
  __shared__ __attribute__((aligned(16))) uint32_t dOp[(BM / 2) * PSTR];
  __shared__ __attribute__((aligned(16))) uint16_t dSs[BM * SSTR];
  __shared__ __attribute__((aligned(16))) uint32_t Kp[(BN / 2) * PSTR];
  __shared__ __attribute__((aligned(16))) float lse_s[BM];
  __shared__ __attribute__((aligned(16))) float dl_s[BM];

  // ---- which (batch, kv head, key tile, split)
  const int per_xcd = gridDim.x >> 3;
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= p.total_wg) return;
  const int per_head = p.kt_total * p.nsplit;
  const int bhk = logical / per_head;
  const int rem = logical - bhk * per_head;
  const int kt = rem / p.nsplit, sp = rem - kt * p.nsplit;
  const int b = bhk / p.Hkv, hk = bhk - b * p.Hkv;
  const int kb = kt >= p.nkt[0] ? 1 : 0;
  const int koff0 = (kb ? kt - p.nkt[0] : kt) * BN;
  const Segment kseg = p.g.k[kb];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hh = lane >> 5;
  const int my_koff = koff0 + 32 * wave + l32;
  const bool key_ok = my_koff < kseg.len;
  const int64_t my_krow = kseg.start + min(my_koff, kseg.len - 1);

  // ---- query tiles that can see this key tile: per q segment, tiles first[qa] .. first[qa]+cnt[qa]-1
  int first[2] = {0, 0}, cnt[2] = {0, 0};
  for (int qa = 0; qa < p.g.nq; ++qa) {
    const int cls = p.g.cls[qa][kb];
    const int nt = (p.g.q[qa].len + BM - 1) / BM;
    if (cls == LOONG_SKIP) continue;
    first[qa] = cls == LOONG_DIAG ? min(koff0 / BM, nt) : 0;
    cnt[qa] = nt - first[qa];
  }
  const int per_g = cnt[0] + cnt[1];
  const int n_it = per_g * p.G;
  const int it_begin = (int)((int64_t)n_it * sp / p.nsplit);
  const int it_end = (int)((int64_t)n_it * (sp + 1) / p.nsplit);

  // ---- K and V rows of this wave as B operands (row my_krow, columns 16ks + 8hh .. +7)
  bf16x8_t kf[NKS], vf[NKS];
  {
    const uint16_t* krow = p.k + b * p.ks[0] + hk * p.ks[1] + my_krow * p.ks[2];
    const uint16_t* vrow = p.v + b * p.ks[0] + hk * p.ks[1] + my_krow * p.ks[2];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      kf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(krow + ks * 16 + hh * 8));
      vf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(vrow + ks * 16 + hh * 8));
    }
  }
  // ---- all 128 keys of the tile, pair-interleaved, for dQ = dS K
  {
    const uint16_t* kbase = p.k + b * p.ks[0] + hk * p.ks[1];
#pragma unroll
    for (int n = 0; n < K_PT; ++n) {
      const int u = tid + n * NT;
      if (K_UNITS % NT == 0 || u < K_UNITS) {
        const int kp = u / CPR, cc = u - kp * CPR;
        const int64_t r0 = kseg.start + min(koff0 + 2 * kp, kseg.len - 1);
        const int64_t r1 = kseg.start + min(koff0 + 2 * kp + 1, kseg.len - 1);
        const uint4 a = *reinterpret_cast<const uint4*>(kbase + r0 * p.ks[2] + cc * 8);
        const uint4 bb = *reinterpret_cast<const uint4*>(kbase + r1 * p.ks[2] + cc * 8);
        uint4 w0, w1;
        interleave_rows(a, bb, w0, w1);
        *reinterpret_cast<uint4*>(&Kp[kp * PSTR + cc * 8]) = w0;
        *reinterpret_cast<uint4*>(&Kp[kp * PSTR + cc * 8 + 4]) = w1;
      }
    }
  }

  floatx16_t dk[NDB], dv[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dk[db][v] = 0.f; dv[db][v] = 0.f; }

  // ---- staging of one Q/dO tile (row pairs) and its row statistics
  uint4 qreg[T_PT][2], oreg[T_PT][2];
  float lse_reg = 0.f, dl_reg = 0.f;
  auto decode = [&](int it, int& h, int& qa, int& i0) {
    const int gq = it / per_g;
    int r = it - gq * per_g;
    qa = r < cnt[0] ? 0 : 1;
    if (qa) r -= cnt[0];
    i0 = (first[qa] + r) * BM;
    h = hk * p.G + gq;
  };
  auto issue_tile = [&](int it) {
    int h, qa, i0;
    decode(it, h, qa, i0);
    const Segment qs = p.g.q[qa];
    const uint16_t* qbase = p.q + b * p.qs[0] + h * p.qs[1];
    const uint16_t* obase = p.d_o + b * p.qs[0] + h * p.qs[1];
#pragma unroll
    for (int n = 0; n < T_PT; ++n) {
      const int u = tid + n * NT;
      if (T_UNITS % NT == 0 || u < T_UNITS) {
        const int ip = u / CPR, cc = u - ip * CPR;
        const int64_t r0 = qs.start + min(i0 + 2 * ip, qs.len - 1), r1 = qs.start + min(i0 + 2 * ip + 1, qs.len - 1);
        qreg[n][0] = *reinterpret_cast<const uint4*>(qbase + r0 * p.qs[2] + cc * 8);
        qreg[n][1] = *reinterpret_cast<const uint4*>(qbase + r1 * p.qs[2] + cc * 8);
        oreg[n][0] = *reinterpret_cast<const uint4*>(obase + r0 * p.qs[2] + cc * 8);
        oreg[n][1] = *reinterpret_cast<const uint4*>(obase + r1 * p.qs[2] + cc * 8);
      }
    }
    if (tid < BM) {
      const int64_t row = ((int64_t)b * p.Hq + h) * p.q_len + qs.start + min(i0 + tid, qs.len - 1);
      const float x = p.lse[row];
      lse_reg = x == -INFINITY ? INFINITY : x * kLog2e;  // a row that saw nothing gets P = 0
      dl_reg = p.delta[row];
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int n = 0; n < T_PT; ++n) {
      const int u = tid + n * NT;
      if (T_UNITS % NT == 0 || u < T_UNITS) {
        const int ip = u / CPR, cc = u - ip * CPR;
        *reinterpret_cast<uint4*>(&Qs[(2 * ip) * RSTR + cc * 8]) = qreg[n][0];
        *reinterpret_cast<uint4*>(&Qs[(2 * ip + 1) * RSTR + cc * 8]) = qreg[n][1];
        *reinterpret_cast<uint4*>(&dOs[(2 * ip) * RSTR + cc * 8]) = oreg[n][0];
        *reinterpret_cast<uint4*>(&dOs[(2 * ip + 1) * RSTR + cc * 8]) = oreg[n][1];
        uint4 w0, w1;
        interleave_rows(qreg[n][0], qreg[n][1], w0, w1);
        *reinterpret_cast<uint4*>(&Qp[ip * PSTR + cc * 8]) = w0;
        *reinterpret_cast<uint4*>(&Qp[ip * PSTR + cc * 8 + 4]) = w1;
        interleave_rows(oreg[n][0], oreg[n][1], w0, w1);
        *reinterpret_cast<uint4*>(&dOp[ip * PSTR + cc * 8]) = w0;
        *reinterpret_cast<uint4*>(&dOp[ip * PSTR + cc * 8 + 4]) = w1;
      }
    }
    if (tid < BM) {
      lse_s[tid] = lse_reg;
      dl_s[tid] = dl_reg;
    }
  };

  if (it_begin < it_end) issue_tile(it_begin);

  for (int it = it_begin; it < it_end; ++it) {
    store_tile();
    __syncthreads();  // tile (and, first time, Kp) visible; previous dQ phase finished
    int h, qa, i0;
    decode(it, h, qa, i0);
    if (it + 1 < it_end) issue_tile(it + 1);
    const Segment qs = p.g.q[qa];
    const bool isdiag = p.g.cls[qa][kb] == LOONG_DIAG;
    const bool need_mask = i0 + BM > qs.len || koff0 + BN > kseg.len || (isdiag && i0 < koff0 + BN - 1);

    // ---- S = Q K^T and dP = dO V^T: rows in registers, one key per lane
    floatx16_t s[NIB], dp[NIB];
#pragma unroll
    for (int ib = 0; ib < NIB; ++ib)
#pragma unroll
      for (int v = 0; v < 16; ++v) { s[ib][v] = 0.f; dp[ib][v] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
      for (int ib = 0; ib < NIB; ++ib) {
        const int off = (ib * 32 + l32) * RSTR + ks * 16 + hh * 8;
        s[ib] = mfma32(as_bf16x8(*reinterpret_cast<const uint4*>(&Qs[off])), kf[ks], s[ib]);
        dp[ib] = mfma32(as_bf16x8(*reinterpret_cast<const uint4*>(&dOs[off])), vf[ks], dp[ib]);
      }

    // ---- P = exp(S - LSE), dS = scale * P * (dP - delta); pack both, dS also to LDS
    uint4 pp[NIB][2], pds[NIB][2];
#pragma unroll
    for (int ib = 0; ib < NIB; ++ib) {
      float pe[16], de[16];
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        const float4 L = *reinterpret_cast<const float4*>(&lse_s[ib * 32 + 8 * vq + 4 * hh]);
        const float4 Dl = *reinterpret_cast<const float4*>(&dl_s[ib * 32 + 8 * vq + 4 * hh]);
        const float Lr[4] = {L.x, L.y, L.z, L.w}, Dr[4] = {Dl.x, Dl.y, Dl.z, Dl.w};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int v = 4 * vq + r;
          float pv = fast_exp2(fmaf(s[ib][v], p.c, -Lr[r]));
          if (need_mask) {
            const int i_off = i0 + ib * 32 + acc_row(v, hh);
            const bool ok = key_ok && i_off < qs.len && (!isdiag || my_koff <= i_off);
            pv = ok ? pv : 0.f;
          }
          pe[v] = pv;
          de[v] = pv * (dp[ib][v] - Dr[r]) * p.scale;
        }
      }
#pragma unroll
      for (int sl = 0; sl < 2; ++sl) {
        pp[ib][sl] = make_uint4(pack_bf16x2(pe[8 * sl + 0], pe[8 * sl + 1]), pack_bf16x2(pe[8 * sl + 2], pe[8 * sl + 3]),
                                pack_bf16x2(pe[8 * sl + 4], pe[8 * sl + 5]), pack_bf16x2(pe[8 * sl + 6], pe[8 * sl + 7]));
        pds[ib][sl] = make_uint4(pack_bf16x2(de[8 * sl + 0], de[8 * sl + 1]), pack_bf16x2(de[8 * sl + 2], de[8 * sl + 3]),
                                 pack_bf16x2(de[8 * sl + 4], de[8 * sl + 5]), pack_bf16x2(de[8 * sl + 6], de[8 * sl + 7]));
      }
      // dS tile, row-major [query row][key]: this lane's key column, 16 rows
#pragma unroll
      for (int sl = 0; sl < 2; ++sl) {
        const uint32_t w[4] = {pds[ib][sl].x, pds[ib][sl].y, pds[ib][sl].z, pds[ib][sl].w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int row = ib * 32 + acc_row(8 * sl + e, hh);
          dSs[row * SSTR + 32 * wave + l32] = (uint16_t)((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xffffu));
        }
      }
    }

    // ---- dV += P^T dO, dK += dS^T Q: contraction over the tile's rows.  Element e of the
    // A operand is row 16*sl + 8*(e/4) + 4*hh + e%4 of block ib, so the B operand takes
    // row pairs 8*sl + {2hh, 2hh+1, 2hh+4, 2hh+5}.
#pragma unroll
    for (int ib = 0; ib < NIB; ++ib)
#pragma unroll
      for (int sl = 0; sl < 2; ++sl) {
        const int base = (ib * 16 + sl * 8 + 2 * hh) * PSTR + l32;
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          uint4 bo, bq;
          bo.x = dOp[base + db * 32]; bo.y = dOp[base + PSTR + db * 32];
          bo.z = dOp[base + 4 * PSTR + db * 32]; bo.w = dOp[base + 5 * PSTR + db * 32];
          dv[db] = mfma32(as_bf16x8(pp[ib][sl]), as_bf16x8(bo), dv[db]);
          bq.x = Qp[base + db * 32]; bq.y = Qp[base + PSTR + db * 32];
          bq.z = Qp[base + 4 * PSTR + db * 32]; bq.w = Qp[base + 5 * PSTR + db * 32];
          dk[db] = mfma32(as_bf16x8(pds[ib][sl]), as_bf16x8(bq), dk[db]);
        }
      }
    __syncthreads();  // dS of all four waves visible

    // ---- dQ tile = dS K over the 128 keys; wave w owns columns 32w .. 32w+31
    if (wave < NDB) {
      floatx16_t dq[NIB];
#pragma unroll
      for (int ib = 0; ib < NIB; ++ib)
#pragma unroll
        for (int v = 0; v < 16; ++v) dq[ib][v] = 0.f;
#pragma unroll
      for (int ksl = 0; ksl < BN / 16; ++ksl) {
        const int kb0 = (8 * ksl + 4 * hh) * PSTR + wave * 32 + l32;
        uint4 bk;
        bk.x = Kp[kb0]; bk.y = Kp[kb0 + PSTR]; bk.z = Kp[kb0 + 2 * PSTR]; bk.w = Kp[kb0 + 3 * PSTR];
#pragma unroll
        for (int ib = 0; ib < NIB; ++ib) {
          const uint4 a = *reinterpret_cast<const uint4*>(&dSs[(ib * 32 + l32) * SSTR + ksl * 16 + hh * 8]);
          dq[ib] = mfma32(as_bf16x8(a), as_bf16x8(bk), dq[ib]);
        }
      }
      float* dq_base = p.dq + b * p.os[0] + h * p.os[1] + wave * 32 + l32;
#pragma unroll
      for (int ib = 0; ib < NIB; ++ib)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int i_off = i0 + ib * 32 + acc_row(v, hh);
          if (i_off < qs.len) unsafeAtomicAdd(dq_base + (int64_t)(qs.start + i_off) * p.os[2], dq[ib][v]);
        }
    }
  }

  // ---- dK, dV of this wave's 32 keys: lane owns one column per block, 16 key rows
  float* dk_base = p.dk + (((int64_t)b * p.Hkv + hk) * p.kv_len + kseg.start) * D + l32;
  float* dv_base = p.dv + (((int64_t)b * p.Hkv + hk) * p.kv_len + kseg.start) * D + l32;
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int koff = koff0 + 32 * wave + acc_row(v, hh);
      if (koff < kseg.len) {
        const int64_t o = (int64_t)koff * D + db * 32;
        if (p.add_dkv) {
          unsafeAtomicAdd(dk_base + o, dk[db][v]);
          unsafeAtomicAdd(dv_base + o, dv[db][v]);
        } else {
          dk_base[o] = dk[db][v];
          dv_base[o] = dv[db][v];
        }
      }
    }
}

__global__ __launch_bounds__(256) void zero_kernel(int64_t n4, float4* a, float4* b) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n4) {
    a[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    b[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
}

template <int D>
int launch_d(BwdParams& p, bool accumulate, hipStream_t st) {
  constexpr int BM = 64, BN = kBwdBN;
  p.kt_total = 0;
  for (int a = 0; a < 2; ++a) {
    p.nkt[a] = a < p.g.nk ? (p.g.k[a].len + BN - 1) / BN : 0;
    p.kt_total += p.nkt[a];
  }
  const int64_t base = (int64_t)p.kt_total * p.Hkv * p.B;
  if (base == 0) return LOONG_OK;
  // spread the query-tile loop over several workgroups when there are few key tiles
  int nsplit = 1;
  if (base < 256) {
    const int64_t q_tiles = (int64_t)p.G * ((p.q_len + BM - 1) / BM);
    nsplit = (int)std::min<int64_t>(std::min<int64_t>((256 + base - 1) / base, 16), std::max<int64_t>(q_tiles, 1));
  }
  p.nsplit = nsplit;
  p.add_dkv = (accumulate || nsplit > 1) ? 1 : 0;
  const int64_t total = base * nsplit;
  if (total > 0x7ffffff0) return fail(LOONG_E_UNSUPPORTED, "backward grid too large");
  p.total_wg = (int)total;
  if (nsplit > 1 && !accumulate) {
    const int64_t n4 = (int64_t)p.B * p.Hkv * p.kv_len * D / 4;
    zero_kernel<<<dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st>>>(n4, reinterpret_cast<float4*>(p.dk),
                                                                          reinterpret_cast<float4*>(p.dv));
    if (int rc = check_launch("loong_attn_step_bwd (clear dk/dv)")) return rc;
  }
  const unsigned grid = (unsigned)((total + 7) / 8 * 8);
  bwd_kernel<D, BM><<<dim3(grid), dim3(kBwdWaves * 64), 0, st>>>(p);
  return check_launch("loong_attn_step_bwd (bf16)");
}

}  // namespace

int launch_bwd_bf16(const loong_step_desc& d, const StepGeom& g, const void* q, const void* k,
                    const void* v, const void* d_o, const float* lse, const float* delta, float* dq,
                    float* dk, float* dv, void* stream) {
  if (d.kv_len == 0) return LOONG_OK;
  BwdParams p{};
  p.q = (const uint16_t*)q; p.k = (const uint16_t*)k; p.v = (const uint16_t*)v; p.d_o = (const uint16_t*)d_o;
  p.lse = lse; p.delta = delta; p.dq = dq; p.dk = dk; p.dv = dv;
  p.B = d.batch; p.Hq = d.n_q_heads; p.Hkv = d.n_kv_heads; p.G = d.n_q_heads / d.n_kv_heads;
  p.q_len = d.q_len; p.kv_len = d.kv_len;
  for (int i = 0; i < 3; ++i) { p.qs[i] = d.q_stride[i]; p.ks[i] = d.kv_stride[i]; p.os[i] = d.o_stride[i]; }
  p.g = g; p.scale = d.softmax_scale; p.c = d.softmax_scale * kLog2e;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool accumulate = d.flags & LOONG_ACCUM_DKV;
  return d.head_dim == 128 ? launch_d<128>(p, accumulate, st) : launch_d<64>(p, accumulate, st);
}

}  // namespace loong
