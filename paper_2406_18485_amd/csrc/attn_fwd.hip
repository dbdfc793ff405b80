// Forward micro-step on bf16 matrix cores: Attention(Q, K, V) of Alg. 2 for the local Q
// chunk against one visiting K/V chunk, with the Update optionally folded in by starting
// the online softmax from the running (out, lse).
//
// Work split.  A workgroup of NW waves owns 32*NW query rows: GS query heads that share
// one kv head (GS | group size) times 32*NW/GS consecutive rows of one zigzag half, so a
// K/V tile staged in LDS serves every head of the group.  Each wave owns 32 rows.
// Per tile of BN keys a wave computes S^T = K Q^T (keys x rows) so that every lane holds
// one query row (two lanes per row, 16 keys each per 32-key block): the row maximum and
// sum are in-lane reductions plus one exchange with the lane 32 places away, and the
// accumulator layout of P^T is already the B-operand layout of the second product
// O^T += V^T P^T, given that V^T is read from LDS with the same key order.
// V is stored in LDS as pairs of keys interleaved per column so that this read is four
// 32-bit loads.  Blocks of the (q half, k half) grid that are invisible are never
// visited; only tiles that touch the diagonal or a ragged end apply a mask.
#include <hip/hip_runtime.h>

#include "device_utils.h"
#include "loong_internal.h"

namespace loong {
namespace {

constexpr float kRescaleSlack = 8.f;  // the running maximum may lag the true one by 2^8

struct FwdParams {
  const uint16_t *q, *k, *v;
  float *out, *lse;
  int B, Hq, Hkv, G, GS;
  int64_t qs[3], ks[3], os[3];
  int q_len;
  StepGeom g;
  float c;         // softmax_scale * log2(e)
  int fuse;
  int ntile[2];    // q tiles per q segment
  int tiles_total;
  int hgroups;     // Hq / GS
  int total_wg;
};

template <int D, int NW, int BN>
struct FwdCfg {
  static constexpr int NT = NW * 64;
  static constexpr int KSTR = D + 8;    // bf16 per K row in LDS (pad: 16-lane b128 reads hit all banks once)
  static constexpr int VSTR = D + 16;   // dwords per key-pair row of V in LDS
  static constexpr int CPR = D / 8;     // 16-byte pieces per row
  static constexpr int K_UNITS = BN * CPR;
  static constexpr int V_UNITS = (BN / 2) * CPR;
  static constexpr int K_PT = (K_UNITS + NT - 1) / NT;
  static constexpr int V_PT = (V_UNITS + NT - 1) / NT;
};

template <int D, int NW, int BN>
__global__ __launch_bounds__(NW * 64) void fwd_kernel(const FwdParams p) {
  using C = FwdCfg<D, NW, BN>;
  constexpr int NJB = BN / 32;  // 32-key blocks per tile
  constexpr int NDB = D / 32;   // 32-column blocks of the output
  constexpr int NKS = D / 16;   // contraction slices of Q K^T
  __shared__ __attribute__((aligned(16))) uint16_t Ks[2][BN * C::KSTR];
  __shared__ __attribute__((aligned(16))) uint32_t Vs[2][(BN / 2) * C::VSTR];

  // ---- which (batch, head group, q tile): consecutive logical ids sit on one XCD, and
  // within a head group the tiles with the most visible keys come first
  const int per_xcd = gridDim.x >> 3;
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= p.total_wg) return;
  const int bh = logical / p.tiles_total;
  const int tt = p.tiles_total - 1 - (logical - bh * p.tiles_total);
  const int b = bh / p.hgroups, hg = bh - b * p.hgroups;
  const int qa = tt >= p.ntile[0] ? 1 : 0;
  const int tile = qa ? tt - p.ntile[0] : tt;
  const int BMH = 32 * NW / p.GS;
  const int row0_wg = tile * BMH;
  const Segment qseg = p.g.q[qa];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hh = lane >> 5;
  const int gq = wave % p.GS, rb = wave / p.GS;
  const int h = hg * p.GS + gq, hk = h / p.G;
  const int wrow0 = row0_wg + rb * 32;
  const int my_off = wrow0 + l32;
  const bool wave_live = wrow0 < qseg.len;
  const bool row_ok = my_off < qseg.len;
  const int my_row = qseg.start + min(my_off, qseg.len - 1);
  const int last_off_wg = min(row0_wg + BMH, qseg.len) - 1;

  // ---- visible key tiles of this workgroup
  int kend[2] = {0, 0}, ntk[2] = {0, 0};
  for (int kb = 0; kb < p.g.nk; ++kb) {
    const int cls = p.g.cls[qa][kb];
    kend[kb] = cls == LOONG_SKIP ? 0 : cls == LOONG_FULL ? p.g.k[kb].len : min(p.g.k[kb].len, last_off_wg + 1);
    ntk[kb] = (kend[kb] + BN - 1) / BN;
  }
  const int total_t = ntk[0] + ntk[1];

  float* out_row = p.out + b * p.os[0] + h * p.os[1] + (int64_t)my_row * p.os[2];
  float* lse_ptr = p.lse + ((int64_t)b * p.Hq + h) * p.q_len + my_row;

  if (total_t == 0) {  // nothing visible: neutral partial result, or leave the running one
    if (!p.fuse && row_ok) {
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq)
          *reinterpret_cast<float4*>(out_row + db * 32 + 8 * vq + 4 * hh) = make_float4(0.f, 0.f, 0.f, 0.f);
      if (hh == 0) *lse_ptr = -INFINITY;
    }
    return;
  }

  // ---- Q fragments (B operand of S^T = K Q^T): row my_row, columns 16*ks + 8*hh .. +7
  bf16x8_t qf[NKS];
  {
    const uint16_t* qrow = p.q + b * p.qs[0] + h * p.qs[1] + (int64_t)my_row * p.qs[2];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(qrow + ks * 16 + hh * 8));
  }

  // ---- running state: maximum (log2 units), partial row sum of this half, O^T accumulators
  float m_run = -INFINITY, l_run = 0.f;
  floatx16_t o[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
  if (p.fuse) {
    const float prev = *lse_ptr;
    if (prev != -INFINITY) {
      m_run = prev * kLog2e;
      l_run = hh == 0 ? 1.f : 0.f;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          const float4 x = *reinterpret_cast<const float4*>(out_row + db * 32 + 8 * vq + 4 * hh);
          o[db][4 * vq + 0] = x.x; o[db][4 * vq + 1] = x.y; o[db][4 * vq + 2] = x.z; o[db][4 * vq + 3] = x.w;
        }
    }
  }

  // ---- global -> register staging of one K/V tile, and register -> LDS
  uint4 kreg[C::K_PT], vreg[C::V_PT][2];
  const uint16_t* kbase = p.k + b * p.ks[0] + hk * p.ks[1];
  const uint16_t* vbase = p.v + b * p.ks[0] + hk * p.ks[1];
  auto tile_of = [&](int t, int& kb, int& j0) {
    kb = t < ntk[0] ? 0 : 1;
    j0 = (t - (kb ? ntk[0] : 0)) * BN;
  };
  auto issue_loads = [&](int t) {
    int kb, j0;
    tile_of(t, kb, j0);
    const int len = p.g.k[kb].len, start = p.g.k[kb].start;
#pragma unroll
    for (int n = 0; n < C::K_PT; ++n) {
      const int u = tid + n * C::NT;
      if (C::K_UNITS % C::NT == 0 || u < C::K_UNITS) {
        const int r = u / C::CPR, cc = u - r * C::CPR;
        const int64_t row = start + min(j0 + r, len - 1);
        kreg[n] = *reinterpret_cast<const uint4*>(kbase + row * p.ks[2] + cc * 8);
      }
    }
#pragma unroll
    for (int n = 0; n < C::V_PT; ++n) {
      const int u = tid + n * C::NT;
      if (C::V_UNITS % C::NT == 0 || u < C::V_UNITS) {
        const int kp = u / C::CPR, cc = u - kp * C::CPR;
        const int64_t r0 = start + min(j0 + 2 * kp, len - 1), r1 = start + min(j0 + 2 * kp + 1, len - 1);
        vreg[n][0] = *reinterpret_cast<const uint4*>(vbase + r0 * p.ks[2] + cc * 8);
        vreg[n][1] = *reinterpret_cast<const uint4*>(vbase + r1 * p.ks[2] + cc * 8);
      }
    }
  };
  auto store_lds = [&](int buf) {
#pragma unroll
    for (int n = 0; n < C::K_PT; ++n) {
      const int u = tid + n * C::NT;
      if (C::K_UNITS % C::NT == 0 || u < C::K_UNITS) {
        const int r = u / C::CPR, cc = u - r * C::CPR;
        *reinterpret_cast<uint4*>(&Ks[buf][r * C::KSTR + cc * 8]) = kreg[n];
      }
    }
#pragma unroll
    for (int n = 0; n < C::V_PT; ++n) {
      const int u = tid + n * C::NT;
      if (C::V_UNITS % C::NT == 0 || u < C::V_UNITS) {
        const int kp = u / C::CPR, cc = u - kp * C::CPR;
        const uint4 a = vreg[n][0], bb = vreg[n][1];  // keys 2kp and 2kp+1, columns 8cc..8cc+7
        uint4 w0, w1;  // dword c = (key 2kp, key 2kp+1) of column 8cc + c
        w0.x = (a.x & 0xffffu) | (bb.x << 16); w0.y = (a.x >> 16) | (bb.x & 0xffff0000u);
        w0.z = (a.y & 0xffffu) | (bb.y << 16); w0.w = (a.y >> 16) | (bb.y & 0xffff0000u);
        w1.x = (a.z & 0xffffu) | (bb.z << 16); w1.y = (a.z >> 16) | (bb.z & 0xffff0000u);
        w1.z = (a.w & 0xffffu) | (bb.w << 16); w1.w = (a.w >> 16) | (bb.w & 0xffff0000u);
        uint32_t* dst = &Vs[buf][kp * C::VSTR + cc * 8];
        *reinterpret_cast<uint4*>(dst) = w0;
        *reinterpret_cast<uint4*>(dst + 4) = w1;
      }
    }
  };

  issue_loads(0);
  store_lds(0);
  __syncthreads();

  for (int t = 0; t < total_t; ++t) {
    const int cur = t & 1;
    if (t + 1 < total_t) issue_loads(t + 1);
    int kb, j0;
    tile_of(t, kb, j0);
    const int klen = p.g.k[kb].len;
    const bool isdiag = p.g.cls[qa][kb] == LOONG_DIAG;
    // a wave whose rows all lie before this tile's first key has nothing to do here
    if (wave_live && !(isdiag && j0 > wrow0 + 31)) {
      // ---- S^T = K Q^T
      floatx16_t s[NJB];
#pragma unroll
      for (int jb = 0; jb < NJB; ++jb)
#pragma unroll
        for (int v = 0; v < 16; ++v) s[jb][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
        for (int jb = 0; jb < NJB; ++jb) {
          const uint4 a = *reinterpret_cast<const uint4*>(&Ks[cur][(jb * 32 + l32) * C::KSTR + ks * 16 + hh * 8]);
          s[jb] = mfma32(as_bf16x8(a), qf[ks], s[jb]);
        }
      // ---- mask (diagonal or ragged end only)
      if (j0 + BN > klen || (isdiag && j0 + BN - 1 > wrow0)) {
#pragma unroll
        for (int jb = 0; jb < NJB; ++jb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int key = j0 + jb * 32 + acc_row(v, hh);
            const bool ok = key < klen && (!isdiag || key <= my_off);
            s[jb][v] = ok ? s[jb][v] : -INFINITY;
          }
      }
      // ---- online softmax with a lagging maximum
      float mx = s[0][0];
#pragma unroll
      for (int jb = 0; jb < NJB; ++jb)
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[jb][v]);
      mx = fmaxf(mx, other_half(mx));
      const float m_cand = mx * p.c;
      if (__builtin_amdgcn_ballot_w64(m_cand > m_run + kRescaleSlack) != 0) {
        const float m_new = fmaxf(m_run, m_cand);
        const float alpha = m_new == -INFINITY ? 1.f : fast_exp2(m_run - m_new);
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
        m_run = m_new;
      }
      const float m_use = m_run == -INFINITY ? 0.f : m_run;
      uint4 pk[NJB][2];
#pragma unroll
      for (int jb = 0; jb < NJB; ++jb) {
        float e[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          e[v] = fast_exp2(fmaf(s[jb][v], p.c, -m_use));
          l_run += e[v];
        }
#pragma unroll
        for (int sl = 0; sl < 2; ++sl)
          pk[jb][sl] = make_uint4(pack_bf16x2(e[8 * sl + 0], e[8 * sl + 1]), pack_bf16x2(e[8 * sl + 2], e[8 * sl + 3]),
                                  pack_bf16x2(e[8 * sl + 4], e[8 * sl + 5]), pack_bf16x2(e[8 * sl + 6], e[8 * sl + 7]));
      }
      // ---- O^T += V^T P^T.  Element e of the B operand is key 16*sl + 8*(e/4) + 4*hh + e%4
      // of block jb, so the A operand takes key pairs 8*sl + {2hh, 2hh+1, 2hh+4, 2hh+5}.
#pragma unroll
      for (int jb = 0; jb < NJB; ++jb)
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) {
          const uint32_t* vp = &Vs[cur][(jb * 16 + sl * 8 + 2 * hh) * C::VSTR + l32];
#pragma unroll
          for (int db = 0; db < NDB; ++db) {
            uint4 a;
            a.x = vp[db * 32];
            a.y = vp[C::VSTR + db * 32];
            a.z = vp[4 * C::VSTR + db * 32];
            a.w = vp[5 * C::VSTR + db * 32];
            o[db] = mfma32(as_bf16x8(a), as_bf16x8(pk[jb][sl]), o[db]);
          }
        }
    }
    if (t + 1 < total_t) store_lds(cur ^ 1);
    __syncthreads();
  }

  // ---- normalise and store
  const float l_tot = l_run + other_half(l_run);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  if (row_ok) {
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq)
        *reinterpret_cast<float4*>(out_row + db * 32 + 8 * vq + 4 * hh) =
            make_float4(o[db][4 * vq] * inv, o[db][4 * vq + 1] * inv, o[db][4 * vq + 2] * inv, o[db][4 * vq + 3] * inv);
    if (hh == 0) *lse_ptr = l_tot > 0.f ? (m_run + fast_log2(l_tot)) * kLn2 : -INFINITY;
  }
}

int pick_gs(int G, int NW) {
  for (int gs = 8; gs >= 1; gs >>= 1)
    if (G % gs == 0 && gs <= NW) return gs;
  return 1;
}

template <int D, int NW, int BN>
int launch_cfg(FwdParams& p, hipStream_t st) {
  p.GS = pick_gs(p.G, NW);
  const int BMH = 32 * NW / p.GS;
  p.tiles_total = 0;
  for (int a = 0; a < 2; ++a) {
    p.ntile[a] = a < p.g.nq ? (p.g.q[a].len + BMH - 1) / BMH : 0;
    p.tiles_total += p.ntile[a];
  }
  p.hgroups = p.Hq / p.GS;
  const int64_t total = (int64_t)p.tiles_total * p.hgroups * p.B;
  if (total == 0) return LOONG_OK;
  if (total > 0x7ffffff0) return fail(LOONG_E_UNSUPPORTED, "forward grid too large");
  p.total_wg = (int)total;
  const unsigned grid = (unsigned)((total + 7) / 8 * 8);
  fwd_kernel<D, NW, BN><<<dim3(grid), dim3(NW * 64), 0, st>>>(p);
  return check_launch("loong_attn_step_fwd (bf16)");
}

}  // namespace

int launch_fwd_bf16(const loong_step_desc& d, const StepGeom& g, const void* q, const void* k,
                    const void* v, float* out, float* lse, void* stream) {
  FwdParams p{};
  p.q = (const uint16_t*)q; p.k = (const uint16_t*)k; p.v = (const uint16_t*)v;
  p.out = out; p.lse = lse;
  p.B = d.batch; p.Hq = d.n_q_heads; p.Hkv = d.n_kv_heads; p.G = d.n_q_heads / d.n_kv_heads;
  for (int i = 0; i < 3; ++i) { p.qs[i] = d.q_stride[i]; p.ks[i] = d.kv_stride[i]; p.os[i] = d.o_stride[i]; }
  p.q_len = d.q_len; p.g = g; p.c = d.softmax_scale * kLog2e; p.fuse = (d.flags & LOONG_FUSE_MERGE) ? 1 : 0;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (d.head_dim == 128) return launch_cfg<128, 8, 64>(p, st);
  return launch_cfg<64, 8, 64>(p, st);
}

}  // namespace loong
