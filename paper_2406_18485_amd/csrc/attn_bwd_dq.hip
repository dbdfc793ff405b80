// dQ pass of the backward micro-step on the 16-bit matrix cores (element class E: bf16 or IEEE
// half; the text below says bf16 for both): this step's share of the
// gradient of the local Q chunk, dQ_i += scale * sum_j dS_ij K_j with
// dS_ij = P_ij (dP_ij - delta_i), P recomputed from the final softmax_lse
// (paper: Sec. 3.1 last paragraph; Alg. 2 run backwards).
//
// The workgroups own query rows, exactly like the forward step: eight waves (two per SIMD)
// = NRB row blocks x KS key splits; a wave keeps the Q and dO fragments of its 32 rows and
// the fp32 dQ^T accumulators in registers while K/V tiles stream through LDS (direct
// global -> LDS loads, XOR-permuted 16-byte pieces, NBUF tiles deep).  Per block of 32 keys:
//   S^T  = K Q^T      A = 16-byte LDS reads of K rows,  B = Q fragments
//   dP^T = V dO^T     A = 16-byte LDS reads of V rows,  B = dO fragments
//   dS^T = P^T o (dP^T - delta)   in registers: a lane holds one query row, so the row's
//                     LSE and delta are per-lane scalars; packed to bf16 it is the B operand of
//   dQ^T += K^T dS^T  A = transposing LDS reads of the same K tile.
// Every row belongs to one wave (after the key splits are summed through LDS), so dQ is
// updated with plain loads and stores in a fixed order: the result is reproducible and no
// atomic traffic goes to L2.
#include <hip/hip_runtime.h>

#include "device_utils.h"
#include "loong_internal.h"
#include "row_tiling.h"
#include "work_map.h"

namespace loong {
namespace {

typedef __attribute__((address_space(3))) void lds_void_t;

struct DqParams {
  const uint16_t *q, *k, *v, *d_o;
  const float *lse, *delta;
  float* dq;
  int B, Hq, Hkv, G, GS;
  int64_t qs[3], ks[3], os[3];
  int q_len;
  StepGeom g;
  float scale, c;  // softmax scale; scale * log2(e)
  int ntile[2];    // q tiles per q segment
  int tiles_total;
  int hgroups;     // Hq / GS
  WorkMap map;     // units = batch x head groups, items = q tiles
};

template <int D, int KS>
struct DqCfg {
  static constexpr int NRB = kRowWaves / KS;       // 32-row blocks per workgroup
  static constexpr int NJB = KS == 1 ? 2 : 1;      // 32-key blocks per wave and iteration
  static constexpr int BNS = 32 * NJB;             // keys per wave and iteration
  static constexpr int TK = KS * BNS;              // keys staged per iteration
  static constexpr int ROWB = D * 2;               // bytes per K or V row
  static constexpr int CH = D / 8;                 // 16-byte pieces per row
  static constexpr int TILE_B = TK * ROWB;         // bytes of one K (or V) tile
  static constexpr int BUF_B = 2 * TILE_B;
  static constexpr int NBUF = BUF_B * 4 <= 131072 ? 4 : 2;
  static constexpr int PD = NBUF - 1;              // tiles in flight ahead of the one being used
  static constexpr int RPI = 1024 / ROWB;          // rows filled by one wave-level load
  static constexpr int KI = TILE_B / 1024 / kRowWaves;  // loads per wave per K (or V) tile
  static constexpr int SLOT_F4 = (D / 32) * 4;     // float4 per lane of one wave's partial result
  static constexpr int TILE_BYTES = NBUF * BUF_B;
  static constexpr int COMB_BYTES = (KS - 1) * NRB * SLOT_F4 * 64 * 16;
  static constexpr int SMEM_BYTES = TILE_BYTES > COMB_BYTES ? TILE_BYTES : COMB_BYTES;
  static_assert(KI >= 1 && KI * 1024 * kRowWaves == TILE_B, "tile must split evenly over the waves");
};

template <class E, int D, int KS>
__global__ __launch_bounds__(kRowWaves * 64) void dq_kernel(const DqParams p) {
  using C = DqCfg<D, KS>;
  constexpr int NRB = C::NRB, NJB = C::NJB, BNS = C::BNS, TK = C::TK, NBUF = C::NBUF, PD = C::PD, KI = C::KI;
  constexpr int NDB = D / 32, NKS = D / 16, ROWB = C::ROWB, CH = C::CH;
  __shared__ __attribute__((aligned(1024))) unsigned char smem[C::SMEM_BYTES];

  // ---- which (batch, head group, q tile): within a head group the tiles with the most
  // visible keys come first
  int bh, rank;
  if (!decode_work(p.map, blockIdx.x, bh, rank)) return;
  const int tt = p.tiles_total - 1 - rank;
  const int b = bh / p.hgroups, hg = bh - b * p.hgroups;
  const int qa = tt >= p.ntile[0] ? 1 : 0;
  const int tile = qa ? tt - p.ntile[0] : tt;
  const int BMH = 32 * NRB / p.GS;
  const int row0_wg = tile * BMH;
  const Segment qseg = qa ? p.g.q[1] : p.g.q[0];

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // in a scalar register: what derives from it stays scalar
  const int rb = wave % NRB, ksp = wave / NRB;  // row block, key split
  const int gq = rb % p.GS, rslot = rb / p.GS;
  const int h = hg * p.GS + gq, hk = h / p.G;
  const int wrow0 = row0_wg + rslot * 32;
  const int my_off = wrow0 + l32;
  const bool wave_live = wrow0 < qseg.len;
  const bool row_ok = my_off < qseg.len;
  const int my_row = qseg.start + min(my_off, qseg.len - 1);
  const int last_off_wg = min(row0_wg + BMH, qseg.len) - 1;

  // ---- visible key tiles of this workgroup (per-segment facts kept in scalars: nothing in
  // the main loop indexes the kernel arguments dynamically)
  const int cls0 = qa ? p.g.cls[1][0] : p.g.cls[0][0];
  const int cls1 = p.g.nk > 1 ? (qa ? p.g.cls[1][1] : p.g.cls[0][1]) : LOONG_SKIP;
  const int klen0 = p.g.k[0].len, klen1 = p.g.nk > 1 ? p.g.k[1].len : 0;
  const int kstart0 = p.g.k[0].start, kstart1 = p.g.nk > 1 ? p.g.k[1].start : 0;
  const int kend0 = cls0 == LOONG_SKIP ? 0 : cls0 == LOONG_FULL ? klen0 : min(klen0, last_off_wg + 1);
  const int kend1 = cls1 == LOONG_SKIP ? 0 : cls1 == LOONG_FULL ? klen1 : min(klen1, last_off_wg + 1);
  const int ntk0 = (kend0 + TK - 1) / TK, ntk1 = (kend1 + TK - 1) / TK;
  const int total_t = ntk0 + ntk1;
  if (total_t == 0) return;  // nothing visible: no share of dQ in this step

  // ---- Q and dO fragments (B operands): row my_row, columns 16 ks + 8 hh .. +7; the row's
  // LSE in log2 units, negated, and its delta.  A row with LSE = -inf sees no key at all.
  bf16x8_t qf[NKS], dof[NKS];
  float nl, dl;
  {
    const int64_t ro = b * p.qs[0] + h * p.qs[1] + (int64_t)my_row * p.qs[2];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      // Q comes with the softmax scale and log2 e folded in (and is rounded to 16 bits again): the
      // score product then ends in the exponent's units and its chain can start from the row's
      // offset (below).  The second rounding moves a recomputed exponent by about 2^-9 of the
      // terms' root sum of squares, a relative change of P well below the 2^-9 that rounding P to
      // 16 bits for the next product costs anyway (the forward pass, whose LSE is compared to
      // 1e-3, keeps the exact multiply-add).
      qf[ks] = scaled_fragment<E>(as_bf16x8(*reinterpret_cast<const uint4*>(p.q + ro + ks * 16 + hh * 8)), p.c);
      dof[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(p.d_o + ro + ks * 16 + hh * 8));
    }
    const int64_t r1 = ((int64_t)b * p.Hq + h) * p.q_len + my_row;
    const float L = p.lse[r1];
    nl = L == -INFINITY ? -INFINITY : L * -kLog2e;
    dl = p.delta[r1];
  }

  floatx16_t ndl;  // -delta of the lane's row in every element: where the dP chains start
  floatx16_t nlt;  // -LSE log2 e of the lane's row in every element: where the score chains start
#pragma unroll
  for (int v = 0; v < 16; ++v) { ndl[v] = -dl; nlt[v] = nl; }
  floatx16_t acc[NDB];  // dQ^T of the wave's rows (without the softmax scale)
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;

  // ---- staging: global -> LDS directly.  Load i of this wave fills LDS bytes
  // [(wave + 8 i) * 1024, +1024) of the K (or V) tile: row (wave + 8 i) * RPI + lane / CH,
  // piece position lane % CH, which holds piece (position ^ swizzle(row)) of that row.
  const unsigned char* kbase = reinterpret_cast<const unsigned char*>(p.k + b * p.ks[0] + hk * p.ks[1]);
  const unsigned char* vbase = reinterpret_cast<const unsigned char*>(p.v + b * p.ks[0] + hk * p.ks[1]);
  const int64_t rowbytes = p.ks[2] * 2;
  const int ld_row = wave * C::RPI + lane / CH;  // row inside the tile for i = 0; later loads add 8*RPI rows
  const uint32_t ld_piece = (uint32_t)((lane % CH) ^ tile_swizzle<D>(ld_row)) * 16;
  const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_void_t*)smem;  // LDS byte address of the buffers
  auto tile_of = [&](int t, int& kb, int& j0) {
    kb = t < ntk0 ? 0 : 1;
    j0 = (t - (kb ? ntk0 : 0)) * TK;
  };
  // byte offsets of this lane's pieces from the first row of a tile (full tiles only; the
  // 32-bit form needs TK rows to span less than 4 GiB, else every tile takes the general path)
  const bool narrow = rowbytes * TK < (int64_t(1) << 32);
  uint32_t ld_off[KI];
#pragma unroll
  for (int i = 0; i < KI; ++i) ld_off[i] = (uint32_t)(ld_row + i * 8 * C::RPI) * (uint32_t)rowbytes + ld_piece;
  auto issue_tile = [&](int t) {
    int kb, j0;
    tile_of(t, kb, j0);
    const int len = kb ? klen1 : klen0, start = kb ? kstart1 : kstart0;
    const int64_t tb = (int64_t)(start + j0) * rowbytes;
    const int last = len - 1 - j0;  // last valid row of the tile (>= 0); later rows repeat it
    const uint32_t kl = smem_base + (t % NBUF) * C::BUF_B + wave * 1024;
    const uint32_t vl = kl + C::TILE_B;
    if (narrow && last >= TK - 1) {  // whole tile: uniform base in scalar registers + per-lane offset
#pragma unroll
      for (int i = 0; i < KI; ++i) {
        load_to_lds_16(kbase + tb, ld_off[i], kl + i * 8192);
        load_to_lds_16(vbase + tb, ld_off[i], vl + i * 8192);
      }
    } else {
#pragma unroll
      for (int i = 0; i < KI; ++i) {
        const int r = min(ld_row + i * 8 * C::RPI, last);
        const int64_t ro = tb + (int64_t)r * rowbytes + ld_piece;
        load_to_lds_16(kbase + ro, kl + i * 8192);
        load_to_lds_16(vbase + ro, vl + i * 8192);
      }
    }
  };

  // ---- LDS read offsets of this lane (bytes inside a tile; the wave's split and the block
  // and slice indices are added as constants: the swizzle repeats every 16 rows)
  // row operand: row l32 (+32 jb), pieces 2 ks + hh
  uint32_t row_rd[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) row_rd[ks] = l32 * ROWB + ((2 * ks + hh) ^ tile_swizzle<D>(l32)) * 16;
  // K^T operand via transposing reads: in a group of 16 lanes, lane i points at row i / 4
  // of a run of four keys and at columns 4 (i % 4) .. +3 of a 16-column strip; it receives
  // the four keys of column i of the strip.  Lanes 0-31 / 32-63 take runs 4 hh .. 4 hh + 3,
  // and the run 8 keys on.
  uint32_t tr_lo[NDB], tr_hi[NDB];
  {
    const int i16 = lane & 15, r = i16 >> 2, qd = i16 & 3, strip = (lane >> 4) & 1;
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      const int piece = db * 4 + strip * 2 + (qd >> 1);
      tr_lo[db] = (4 * hh + r) * ROWB + (piece ^ tile_swizzle<D>(4 * hh + r)) * 16 + (qd & 1) * 8;
      tr_hi[db] = (4 * hh + r + 8) * ROWB + (piece ^ tile_swizzle<D>(4 * hh + r + 8)) * 16 + (qd & 1) * 8;
    }
  }

  // ---- pipeline: PD tiles in flight.  Everything loaded so far is waited for here, so that
  // no counter wait of the compiler's own ends up inside the loop, where it would also wait
  // for the tiles in flight.
  wait_vmcnt<0>();
#pragma unroll
  for (int t = 0; t < PD; ++t)
    if (t < total_t) issue_tile(t);

  for (int t = 0; t < total_t; ++t) {
    // this wave's loads of tile t have landed when at most the later tiles' are outstanding
    const int later = min(PD - 1, total_t - 1 - t);
    if (later >= 2) wait_vmcnt<2 * 2 * KI>();
    else if (later == 1) wait_vmcnt<2 * KI>();
    else wait_vmcnt<0>();
    __syncthreads();  // every wave's part of tile t is in LDS; everyone has finished tile t-1
    if (t + PD < total_t) issue_tile(t + PD);  // into the buffer tile t-1 used

    int kb, jt;
    tile_of(t, kb, jt);
    const int klen = kb ? klen1 : klen0;
    const bool isdiag = (kb ? cls1 : cls0) == LOONG_DIAG;
    const unsigned char* Kt = smem + (t % NBUF) * C::BUF_B + ksp * BNS * ROWB;
    const unsigned char* Vt = Kt + C::TILE_B;

#pragma unroll
    for (int jb = 0; jb < NJB; ++jb) {
      // A wave skips a block whose keys lie past the end of the segment or past all of its rows.
      const int j0 = jt + ksp * BNS + jb * 32;
      if (!wave_live || j0 >= klen || (isdiag && j0 > wrow0 + 31)) continue;
      const unsigned char* Kb = Kt + jb * 32 * ROWB;
      const unsigned char* Vb = Vt + jb * 32 * ROWB;

      // ---- S^T = K Q^T, dP^T = V dO^T (keys x rows: a lane holds one query row).  The K and V
      // row operands are requested PF products ahead (in program order, held there by the
      // scheduling barriers): left to itself the compiler keeps two reads in flight and every
      // pair of products then waits out a full LDS latency.
      floatx16_t s, dp;
      {
        constexpr int NIT = 2 * NKS, PF = 4;
        auto row_frag = [&](int it) {
          return as_bf16x8(*reinterpret_cast<const uint4*>(((it & 1) ? Vb : Kb) + row_rd[it >> 1]));
        };
        bf16x8_t ring[PF + 1];
        static_for<0, PF>([&](auto i) { ring[i.value] = row_frag(i.value); });
        // (the dP chain starts from -delta of the lane's row, so it ends as dP - delta; the score
        // chain from -LSE log2 e, so it ends as the exponent of P: two vector instructions per
        // element that the matrix cores do on the side)
        static_for<0, NIT>([&](auto i) {
          constexpr int it = i.value, ks = it >> 1;
          if constexpr (it + PF < NIT) ring[(it + PF) % (PF + 1)] = row_frag(it + PF);
          __builtin_amdgcn_sched_barrier(0);
          if constexpr (it & 1) dp = E::mfma(ring[it % (PF + 1)], dof[ks], ks ? dp : ndl);
          else s = E::mfma(ring[it % (PF + 1)], qf[ks], ks ? s : nlt);
        });
      }
      // ---- dS^T = P^T (dP^T - delta), the softmax scale is applied to the sums at the end
      float e[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) e[v] = fast_exp2(s[v]) * dp[v];
      if (j0 + 32 > klen || (isdiag && j0 + 31 > wrow0)) {  // diagonal or ragged end only
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = j0 + acc_row(v, hh);
          const bool ok = key < klen && (!isdiag || key <= my_off);
          e[v] = ok ? e[v] : 0.f;
        }
      }
      uint4 pk[2];
#pragma unroll
      for (int sl = 0; sl < 2; ++sl)
        pk[sl] = make_uint4(E::pack2(e[8 * sl + 0], e[8 * sl + 1]), E::pack2(e[8 * sl + 2], e[8 * sl + 3]),
                            E::pack2(e[8 * sl + 4], e[8 * sl + 5]), E::pack2(e[8 * sl + 6], e[8 * sl + 7]));
      // ---- dQ^T += K^T dS^T.  Element e of the B operand is key 16 sl + 8 (e / 4) + 4 hh + e % 4
      // of the block: the A operand is the run starting at key 16 sl + 4 hh and the run 8 keys on.
#pragma unroll
      for (int sl = 0; sl < 2; ++sl)
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          const unsigned char* kp = Kb + sl * 16 * ROWB;
          acc[db] = E::mfma(read_tr_pair(kp + tr_lo[db], kp + tr_hi[db]), as_bf16x8(pk[sl]), acc[db]);
        }
    }
  }

  // ---- sum the key splits: splits 1.. park their dQ^T in LDS, split 0 adds them in order.
  // Split 0 requests its rows of dQ first: the round trip to memory runs while the others park.
  float* const dq_row = p.dq + b * p.os[0] + h * p.os[1] + (int64_t)my_row * p.os[2];
  float4 old[NDB][4];
  if (KS > 1) {
    if (ksp == 0 && row_ok) {
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) old[db][vq] = *reinterpret_cast<const float4*>(dq_row + db * 32 + 8 * vq + 4 * hh);
    }
    __syncthreads();  // all reads of the last tile are done: the tile buffers are reused
    float4* slots = reinterpret_cast<float4*>(smem);
    if (ksp > 0) {
      float4* mine = slots + ((ksp - 1) * NRB + rb) * C::SLOT_F4 * 64 + lane;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq)
          mine[(db * 4 + vq) * 64] = make_float4(acc[db][4 * vq], acc[db][4 * vq + 1], acc[db][4 * vq + 2], acc[db][4 * vq + 3]);
    }
    __syncthreads();
    if (ksp > 0) return;
#pragma unroll 1
    for (int sp = 1; sp < KS; ++sp) {
      const float4* theirs = slots + ((sp - 1) * NRB + rb) * C::SLOT_F4 * 64 + lane;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          const float4 x = theirs[(db * 4 + vq) * 64];
          acc[db][4 * vq + 0] += x.x; acc[db][4 * vq + 1] += x.y;
          acc[db][4 * vq + 2] += x.z; acc[db][4 * vq + 3] += x.w;
        }
    }
  }

  // ---- dQ row += scale * sum: register 4 vq + r of block db is column 32 db + 8 vq + 4 hh + r
  if (row_ok) {
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        float4* dst = reinterpret_cast<float4*>(dq_row + db * 32 + 8 * vq + 4 * hh);
        float4 x = KS > 1 ? old[db][vq] : *dst;
        x.x = fmaf(acc[db][4 * vq + 0], p.scale, x.x); x.y = fmaf(acc[db][4 * vq + 1], p.scale, x.y);
        x.z = fmaf(acc[db][4 * vq + 2], p.scale, x.z); x.w = fmaf(acc[db][4 * vq + 3], p.scale, x.w);
        *dst = x;
      }
  }
}

template <class E, int D, int KS>
int launch_cfg(DqParams& p, hipStream_t st) {
  const RowTiling rt = make_row_tiling(p.g, p.G, p.Hq, p.B, kRowWaves / KS, /*list_blind=*/false);
  p.GS = rt.GS; p.ntile[0] = rt.ntile[0]; p.ntile[1] = rt.ntile[1];
  p.tiles_total = rt.tiles_total; p.hgroups = rt.hgroups;
  if (rt.total_wg == 0) return LOONG_OK;
  if (rt.total_wg > 0x3ffffff0) return fail(LOONG_E_UNSUPPORTED, "backward (dQ) grid too large");
  p.map = make_work_map((int64_t)p.B * rt.hgroups, rt.tiles_total);
  dq_kernel<E, D, KS><<<dim3(p.map.grid), dim3(kRowWaves * 64), 0, st>>>(p);
  return check_launch("loong_attn_step_bwd (bf16, dQ)");
}

template <class E>
int pick_cfg(DqParams& p, int head_dim, int ks, hipStream_t st) {
  if (head_dim == 128) {
    if (ks == 1) return launch_cfg<E, 128, 1>(p, st);
    if (ks == 2) return launch_cfg<E, 128, 2>(p, st);
    return launch_cfg<E, 128, 4>(p, st);
  }
  if (ks == 1) return launch_cfg<E, 64, 1>(p, st);
  if (ks == 2) return launch_cfg<E, 64, 2>(p, st);
  return launch_cfg<E, 64, 4>(p, st);
}

}  // namespace

int launch_bwd_dq_bf16(const loong_step_desc& d, const StepGeom& g, const void* q, const void* k,
                       const void* v, const void* d_o, const float* lse, const float* delta, float* dq,
                       void* stream) {
  if (d.kv_len == 0 || d.q_len == 0) return LOONG_OK;
  DqParams p{};
  p.q = (const uint16_t*)q; p.k = (const uint16_t*)k; p.v = (const uint16_t*)v; p.d_o = (const uint16_t*)d_o;
  p.lse = lse; p.delta = delta; p.dq = dq;
  p.B = d.batch; p.Hq = d.n_q_heads; p.Hkv = d.n_kv_heads; p.G = d.n_q_heads / d.n_kv_heads;
  for (int i = 0; i < 3; ++i) { p.qs[i] = d.q_stride[i]; p.ks[i] = d.kv_stride[i]; p.os[i] = d.o_stride[i]; }
  p.q_len = d.q_len; p.g = g; p.scale = d.softmax_scale; p.c = d.softmax_scale * kLog2e;
  hipStream_t st = static_cast<hipStream_t>(stream);
  DeviceFacts dev;
  if (int rc = device_facts(&dev)) return rc;
  const int ks = pick_key_splits(g, p.G, p.Hq, p.B, forced_key_splits(d.flags), dev.cus);
  if (d.dtype == LOONG_FP16) return pick_cfg<Fp16>(p, d.head_dim, ks, st);
  return pick_cfg<Bf16>(p, d.head_dim, ks, st);
}

}  // namespace loong
