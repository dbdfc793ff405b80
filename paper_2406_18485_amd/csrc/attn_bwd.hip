// Backward micro-step on bf16 matrix cores: gradients of the visiting K/V chunk and this
// step's share of dQ, recomputing the probabilities from the final softmax_lse
// (paper: Sec. 3.1 last paragraph; Sec. "Selective Checkpoint++").
//
// Work split.  A workgroup of 4 waves (one per SIMD, up to 512 registers each) owns 128 keys
// of one kv head, 32 per wave, and walks over the 64-row query tiles of every q head of
// the group that can see them.  Loop-invariant in registers: the wave's K and V rows as B
// operands of S = Q K^T and dP = dO V^T, the K columns it needs for dQ, and the fp32
// dK / dV accumulators.
//
// Per query tile: Q, dO (row-major) and the rows' LSE and delta go from global memory
// straight into LDS, one tile ahead, with the 16-byte pieces of every row XOR-permuted so
// that both kinds of LDS read below are free of bank conflicts.
//   S, dP     A operand = 16-byte reads of Q / dO rows; accumulators put one key per lane
//             and 16 query rows per 32x32 block in registers;
//   dV, dK    contraction over rows: A operand = P^T / dS^T straight from those
//             accumulators, B operand = transposing LDS reads of the same dO / Q tiles;
//   dQ        contraction over keys: dS^T is written to LDS once ([key][row], 8-byte
//             stores), read back with transposing reads as the A operand, B operand = the
//             K columns in registers; each wave adds a 32 x 64 (or 32 x 32) piece of the
//             dQ tile to global memory with fp32 atomics.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <type_traits>

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
constexpr int kBwdBN = 32 * kBwdWaves;  // keys per workgroup
constexpr int kBwdBM = 64;              // query rows per iteration

template <int D, bool WITH_DQ>
struct BwdCfg {
  static constexpr int BM = kBwdBM, BN = kBwdBN;
  static constexpr int ROWB = D * 2;               // bytes per row of a Q / dO / K tile
  static constexpr int CH = D / 8;                 // 16-byte pieces per row
  static constexpr int RPI = 1024 / ROWB;          // rows filled by one wave-level load
  static constexpr int QT_B = BM * ROWB;           // bytes of a Q (or dO) tile
  static constexpr int LI = QT_B / 1024 / kBwdWaves;  // loads per wave per Q (or dO) tile
  static constexpr int STAGE_B = 2 * QT_B + 2 * BM * 4;  // Q, dO, lse, delta
  static constexpr int DS_STR = BM * 2 + 16;       // bytes per key row of the dS^T tile (padded)
  static constexpr int DS_B = WITH_DQ ? BN * DS_STR : 0;
  static constexpr int KT_B = BN * ROWB;           // K tile staged once for the transposed fragments
  static constexpr int STAGES_B = (2 * STAGE_B > KT_B || !WITH_DQ) ? 2 * STAGE_B : KT_B;
  static constexpr int SMEM_BYTES = STAGES_B + DS_B;
  static constexpr int NDQ = D / 64;               // 32-column blocks of dQ per wave
};

template <int D, bool WITH_DQ>
__global__ __launch_bounds__(kBwdWaves * 64) void bwd_kernel(const BwdParams p) {
  using C = BwdCfg<D, WITH_DQ>;
  constexpr int BM = C::BM, BN = C::BN, ROWB = C::ROWB, CH = C::CH, LI = C::LI, NDQ = C::NDQ;
  constexpr int NKS = D / 16, NDB = D / 32, NIB = BM / 32, NKSL = BN / 16;
  __shared__ __attribute__((aligned(1024))) unsigned char smem[C::SMEM_BYTES];
  unsigned char* const dst_lds = smem + C::STAGES_B;  // dS^T tile

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
  const Segment kseg = kb ? p.g.k[1] : p.g.k[0];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hh = lane >> 5;
  const int my_koff = koff0 + 32 * wave + l32;
  const bool key_ok = my_koff < kseg.len;
  const int64_t my_krow = kseg.start + min(my_koff, kseg.len - 1);

  // ---- query tiles that can see this key tile: per q segment, tiles first .. first + cnt - 1
  // (per-segment facts in scalars: the loop never indexes the kernel arguments dynamically)
  const int clsq0 = kb ? p.g.cls[0][1] : p.g.cls[0][0];
  const int clsq1 = p.g.nq > 1 ? (kb ? p.g.cls[1][1] : p.g.cls[1][0]) : LOONG_SKIP;
  const int qlen0 = p.g.q[0].len, qlen1 = p.g.nq > 1 ? p.g.q[1].len : 0;
  const int qstart0 = p.g.q[0].start, qstart1 = p.g.nq > 1 ? p.g.q[1].start : 0;
  const int nt0 = (qlen0 + BM - 1) / BM, nt1 = (qlen1 + BM - 1) / BM;
  const int first0 = clsq0 == LOONG_DIAG ? min(koff0 / BM, nt0) : 0;
  const int first1 = clsq1 == LOONG_DIAG ? min(koff0 / BM, nt1) : 0;
  const int cnt0 = clsq0 == LOONG_SKIP ? 0 : nt0 - first0;
  const int cnt1 = clsq1 == LOONG_SKIP ? 0 : nt1 - first1;
  const int per_g = cnt0 + cnt1;
  const int n_it = per_g * p.G;
  const int it_begin = (int)((int64_t)n_it * sp / p.nsplit);
  const int it_end = (int)((int64_t)n_it * (sp + 1) / p.nsplit);
  auto decode = [&](int it, int& h, int& qa, int& i0) {
    const int gq = it / per_g;
    int r = it - gq * per_g;
    qa = r < cnt0 ? 0 : 1;
    if (qa) r -= cnt0;
    i0 = ((qa ? first1 : first0) + r) * BM;
    h = hk * p.G + gq;
  };

  // ---- K and V rows of this wave as B operands (row my_krow, columns 16 ks + 8 hh .. +7)
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

  // ---- per-lane pieces of the staging and of the LDS reads
  const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;
  // direct loads: load i of this wave fills LDS bytes [(wave + 4 i) * 1024, +1024) of a tile
  const int ld_row = wave * C::RPI + lane / CH;  // row inside the tile for i = 0; later loads add 4 * RPI rows
  const uint32_t ld_piece = (uint32_t)((lane % CH) ^ tile_swizzle<D>(ld_row)) * 16;
  // A operand of S / dP: row l32 (+32 ib), pieces 2 ks + hh
  uint32_t row_rd[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) row_rd[ks] = l32 * ROWB + ((2 * ks + hh) ^ tile_swizzle<D>(l32)) * 16;
  // transposing reads of a row-major tile: run of four rows starting at 4 hh (+8 for the
  // second run; +16 sl, +32 ib as constants), 16-column strip (lane >> 4) & 1 of block db
  const int i16 = lane & 15, tr_r = i16 >> 2, tr_q = i16 & 3, strip = (lane >> 4) & 1;
  uint32_t tr_lo[NDB], tr_hi[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) {
    const int piece = db * 4 + strip * 2 + (tr_q >> 1);
    tr_lo[db] = (4 * hh + tr_r) * ROWB + (piece ^ tile_swizzle<D>(4 * hh + tr_r)) * 16 + (tr_q & 1) * 8;
    tr_hi[db] = (4 * hh + tr_r + 8) * ROWB + (piece ^ tile_swizzle<D>(4 * hh + tr_r + 8)) * 16 + (tr_q & 1) * 8;
  }
  // transposing reads of the dS^T tile ([key][row], padded rows): key run 4 hh + r (+8),
  // rows (columns of the tile) 16 strip + 4 q .. +3 of block ib
  const uint32_t ds_rd = (4 * hh + tr_r) * C::DS_STR + (strip * 16 + tr_q * 4) * 2;

  // dQ atomics: 32-bit offsets of this lane's 16 accumulator rows from the tile's first element
  uint32_t dq_off[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) dq_off[v] = (uint32_t)(acc_row(v, hh) * p.os[2] + l32) * 4;

  // ---- the K columns this wave needs for dQ, as B operands [key][column] with the keys of
  // every 16-key slice in accumulator order: staged once through LDS, read transposed
  const int dq_ib = wave & 1, dq_db0 = (wave >> 1) * NDQ;  // this wave's piece of the dQ tile
  bf16x8_t ktf[NDQ][NKSL];
  if constexpr (WITH_DQ) {
    const unsigned char* kbase = reinterpret_cast<const unsigned char*>(p.k + b * p.ks[0] + hk * p.ks[1]);
    const int64_t rowbytes = p.ks[2] * 2;
    const int last = kseg.len - 1 - koff0;
#pragma unroll
    for (int i = 0; i < C::KT_B / 1024 / kBwdWaves; ++i) {
      const int r = min(ld_row + i * 4 * C::RPI, last);
      load_to_lds_16(kbase + (int64_t)(kseg.start + koff0 + r) * rowbytes + ld_piece, smem_base + (wave + 4 * i) * 1024);
    }
    wait_vmcnt<0>();
    __syncthreads();
#pragma unroll
    for (int n = 0; n < NDQ; ++n)
#pragma unroll
      for (int ksl = 0; ksl < NKSL; ++ksl)
        ktf[n][ksl] = read_tr_pair(smem + ksl * 16 * ROWB + tr_lo[dq_db0 + n], smem + ksl * 16 * ROWB + tr_hi[dq_db0 + n]);
    __syncthreads();  // the staging area is reused for the query tiles
  }

  floatx16_t dk[NDB], dv[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dk[db][v] = 0.f; dv[db][v] = 0.f; }

  // ---- staging of one query tile: Q, dO rows and their LSE / delta, global -> LDS
  auto issue_tile = [&](int it) {
    int h, qa, i0;
    decode(it, h, qa, i0);
    const int qlen = qa ? qlen1 : qlen0, qstart = qa ? qstart1 : qstart0;
    const int last = qlen - 1 - i0;
    const uint32_t st = smem_base + (it & 1) * C::STAGE_B;
    const unsigned char* qb = reinterpret_cast<const unsigned char*>(p.q + b * p.qs[0] + h * p.qs[1]);
    const unsigned char* ob = reinterpret_cast<const unsigned char*>(p.d_o + b * p.qs[0] + h * p.qs[1]);
    const int64_t rowbytes = p.qs[2] * 2;
#pragma unroll
    for (int i = 0; i < LI; ++i) {
      const int r = min(ld_row + i * 4 * C::RPI, last);
      const int64_t ro = (int64_t)(qstart + i0 + r) * rowbytes + ld_piece;
      load_to_lds_16(qb + ro, st + (wave + 4 * i) * 1024);
      load_to_lds_16(ob + ro, st + C::QT_B + (wave + 4 * i) * 1024);
    }
    if (wave < 2) {  // wave 0: the 64 rows' LSE, wave 1: their delta
      const int64_t row = ((int64_t)b * p.Hq + h) * p.q_len + qstart + i0 + min(lane, last);
      load_to_lds_4((wave ? p.delta : p.lse) + row, st + 2 * C::QT_B + wave * BM * 4);
    }
  };

  wait_vmcnt<0>();  // K / V fragments are in: no counter wait of the compiler's lands in the loop
  if (it_begin < it_end) issue_tile(it_begin);
  wait_vmcnt<0>();

  for (int it = it_begin; it < it_end; ++it) {
    __syncthreads();  // tile `it` is in LDS (each wave waited for its part); iteration it - 1 is finished
    if (it + 1 < it_end) issue_tile(it + 1);
    int h, qa, i0;
    decode(it, h, qa, i0);
    const int qlen = qa ? qlen1 : qlen0, qstart = qa ? qstart1 : qstart0;
    const bool isdiag = (qa ? clsq1 : clsq0) == LOONG_DIAG;
    const bool need_mask = i0 + BM > qlen || koff0 + BN > kseg.len || (isdiag && i0 < koff0 + BN - 1);
    const unsigned char* Qt = smem + (it & 1) * C::STAGE_B;
    const unsigned char* Ot = Qt + C::QT_B;
    const float* lse_s = reinterpret_cast<const float*>(Qt + 2 * C::QT_B);
    const float* dl_s = lse_s + BM;

    // ---- S = Q K^T and dP = dO V^T: rows in registers, one key per lane
    floatx16_t s[NIB], dp[NIB];
    {
      floatx16_t zero;
#pragma unroll
      for (int v = 0; v < 16; ++v) zero[v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
        for (int ib = 0; ib < NIB; ++ib) {
          s[ib] = mfma32(as_bf16x8(*reinterpret_cast<const uint4*>(Qt + ib * 32 * ROWB + row_rd[ks])), kf[ks], ks ? s[ib] : zero);
          dp[ib] = mfma32(as_bf16x8(*reinterpret_cast<const uint4*>(Ot + ib * 32 * ROWB + row_rd[ks])), vf[ks], ks ? dp[ib] : zero);
        }
    }

    // ---- P = exp(S - LSE), dS = scale * P * (dP - delta); pack both; dS^T to LDS.
    // (A row whose LSE is -inf sees no key in any step: such pairs are always masked.)
    uint4 pp[NIB][2], pds[NIB][2];
    auto probabilities = [&](auto masked) {
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
            float pv = fast_exp2(fmaf(s[ib][v], p.c, Lr[r] * -kLog2e));
            if (decltype(masked)::value) {
              const int i_off = i0 + ib * 32 + acc_row(v, hh);
              const bool ok = key_ok && i_off < qlen && (!isdiag || my_koff <= i_off);
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
          // dS^T tile, [key][row]: this lane's key row, rows acc_row(8 sl + 0..3) and (8 sl + 4..7)
          if constexpr (WITH_DQ) {
            unsigned char* drow = dst_lds + (32 * wave + l32) * C::DS_STR + (ib * 32 + 16 * sl + 4 * hh) * 2;
            *reinterpret_cast<uint2*>(drow) = make_uint2(pds[ib][sl].x, pds[ib][sl].y);
            *reinterpret_cast<uint2*>(drow + 16) = make_uint2(pds[ib][sl].z, pds[ib][sl].w);
          }
        }
      }
    };
    if (need_mask) probabilities(std::true_type{});
    else probabilities(std::false_type{});

    // ---- dV += P^T dO, dK += dS^T Q: contraction over the tile's rows.  Element e of the A
    // operand is row 16 sl + 8 (e / 4) + 4 hh + e % 4 of block ib: the B operand is the run
    // of four rows starting at 16 sl + 4 hh and the run 8 rows on.
#pragma unroll
    for (int ib = 0; ib < NIB; ++ib)
#pragma unroll
      for (int sl = 0; sl < 2; ++sl)
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          const int ro = (ib * 32 + sl * 16) * ROWB;
          dv[db] = mfma32(as_bf16x8(pp[ib][sl]), read_tr_pair(Ot + ro + tr_lo[db], Ot + ro + tr_hi[db]), dv[db]);
          dk[db] = mfma32(as_bf16x8(pds[ib][sl]), read_tr_pair(Qt + ro + tr_lo[db], Qt + ro + tr_hi[db]), dk[db]);
        }
    if constexpr (!WITH_DQ) {
      wait_vmcnt<0>();  // this wave's part of the next tile, issued a whole iteration ago
      continue;
    }
    __syncthreads();  // dS^T of all four waves visible

    // ---- dQ tile = dS K over the 128 keys; this wave: rows 32 dq_ib .., columns 32 dq_db0 ..
    floatx16_t dq[NDQ];
#pragma unroll
    for (int n = 0; n < NDQ; ++n)
#pragma unroll
      for (int v = 0; v < 16; ++v) dq[n][v] = 0.f;
#pragma unroll
    for (int ksl = 0; ksl < NKSL; ++ksl) {
      const unsigned char* ap = dst_lds + ksl * 16 * C::DS_STR + dq_ib * 64 + ds_rd;
      const bf16x8_t a = read_tr_pair(ap, ap + 8 * C::DS_STR);
#pragma unroll
      for (int n = 0; n < NDQ; ++n) dq[n] = mfma32(a, ktf[n][ksl], dq[n]);
    }
    // The next tile's loads were issued a whole iteration ago: wait for them here, before the
    // atomics, which share the counter with them and complete in no fixed order; nothing
    // ever waits for the atomics.
    wait_vmcnt<0>();
    unsigned char* dq_tile = reinterpret_cast<unsigned char*>(
        p.dq + b * p.os[0] + h * p.os[1] + (int64_t)(qstart + i0 + dq_ib * 32) * p.os[2] + dq_db0 * 32);
    if (i0 + BM <= qlen) {
#pragma unroll
      for (int n = 0; n < NDQ; ++n)
#pragma unroll
        for (int v = 0; v < 16; ++v) unsafeAtomicAdd(reinterpret_cast<float*>(dq_tile + dq_off[v]) + n * 32, dq[n][v]);
    } else {
#pragma unroll
      for (int n = 0; n < NDQ; ++n)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (i0 + dq_ib * 32 + acc_row(v, hh) < qlen)
            unsafeAtomicAdd(reinterpret_cast<float*>(dq_tile + dq_off[v]) + n * 32, dq[n][v]);
    }
  }

  // ---- dK (times the softmax scale's share already in dS), dV of this wave's 32 keys:
  // a lane owns one column per block and 16 key rows
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
int launch_d(BwdParams& p, bool accumulate, bool with_dq, hipStream_t st) {
  constexpr int BM = kBwdBM, BN = kBwdBN;
  p.kt_total = 0;
  for (int a = 0; a < 2; ++a) {
    p.nkt[a] = a < p.g.nk ? (p.g.k[a].len + BN - 1) / BN : 0;
    p.kt_total += p.nkt[a];
  }
  const int64_t base = (int64_t)p.kt_total * p.Hkv * p.B;
  if (base == 0) return LOONG_OK;
  // Key tiles that some query can see; the query-tile loop is spread over several workgroups
  // when those are fewer than the CUs, and once more when a diagonal block makes their
  // loop lengths uneven.
  int64_t busy = 0;
  bool diag = false;
  for (int kb = 0; kb < p.g.nk; ++kb) {
    bool seen = false;
    for (int a = 0; a < p.g.nq; ++a) {
      seen |= p.g.cls[a][kb] != LOONG_SKIP && p.g.q[a].len > 0;
      diag |= p.g.cls[a][kb] == LOONG_DIAG;
    }
    if (seen) busy += p.nkt[kb];
  }
  busy *= (int64_t)p.Hkv * p.B;
  int nsplit = 1;
  const int64_t q_tiles = std::max<int64_t>((int64_t)p.G * ((p.q_len + BM - 1) / BM), 1);
  if (busy > 0 && busy < 256) nsplit = (int)std::min<int64_t>((256 + busy - 1) / busy, 16);
  if (diag && busy * nsplit <= 512) nsplit *= 2;
  nsplit = (int)std::min<int64_t>(nsplit, q_tiles);
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
  if (with_dq) bwd_kernel<D, true><<<dim3(grid), dim3(kBwdWaves * 64), 0, st>>>(p);
  else bwd_kernel<D, false><<<dim3(grid), dim3(kBwdWaves * 64), 0, st>>>(p);
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
  // dQ either from the same kernel (fp32 atomics) or from the row-owning pass that follows.
  // LOONG_BWD_DQ=atomic selects the former (tuning aid).
  const char* mode = std::getenv("LOONG_BWD_DQ");
  const bool fused_dq = mode && std::strcmp(mode, "atomic") == 0;
  const int rc = d.head_dim == 128 ? launch_d<128>(p, accumulate, fused_dq, st) : launch_d<64>(p, accumulate, fused_dq, st);
  if (rc != LOONG_OK || fused_dq) return rc;
  return launch_bwd_dq_bf16(d, g, q, k, v, d_o, lse, delta, dq, stream);
}

}  // namespace loong
