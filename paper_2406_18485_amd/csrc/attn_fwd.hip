// Forward micro-step on the 16-bit matrix cores (element class E: bf16 or IEEE half; the text
// below says bf16 for both): Attention(Q, K, V) of Alg. 2 for the local Q
// chunk against one visiting K/V chunk, with the Update optionally folded in by starting
// the online softmax from the running (out, lse).
//
// Shape of the computation.  A workgroup has eight waves (two per SIMD) = NRB row blocks
// x KS key splits.  Every wave owns 32 query rows of one head and keeps their Q fragments
// and fp32 O^T accumulators in registers.  Per iteration a tile of KS*BNS keys is staged
// in LDS and the wave takes its BNS keys: S^T = K Q^T (keys x rows) with
// v_mfma_f32_32x32x16_bf16, so a lane holds one query row (row maximum and sum are in-lane
// reductions plus one exchange with the lane 32 places away) and the accumulator layout of
// P^T already is the B operand of O^T += V^T P^T.
//
// Staging.  K and V tiles go from global memory straight into LDS (global_load_lds, 16 B
// per lane, no registers, no LDS writes by the waves), row-major as in memory, NBUF tiles
// deep.  Each wave-level load fills 1 KB of LDS contiguously, so the rows cannot be padded;
// bank conflicts are avoided by permuting which 16-byte piece of a row each lane fetches
// (an XOR of the piece index with low bits of the row; the LDS serves 256 bytes per clock,
// i.e. 16 lanes of a 16-byte read or 32 lanes of a transposing read, and the XORs make each
// such group touch every bank once).  K operands are then single
// 16-byte LDS reads; V^T operands are two transposing reads (ds_read_b64_tr_b16), each
// giving a lane four consecutive keys of one column: exactly the two runs of four keys a
// lane holds per 16-key slice of the P^T accumulator.
//
// Work split.  With KS = 1 eight waves (256 rows, or GS heads of one kv group x 256/GS
// rows) share each staged tile.  When a step has too few rows to fill the chip, KS = 2 or
// 4 waves share the same rows and split every tile's keys, each with its own online
// softmax; the partial results are combined through LDS at the end (the log-sum-exp
// algebra of Update).  Blocks of the (q half, k half) grid that are invisible are never
// visited; only tiles touching the diagonal or a ragged end apply a mask.
#include <hip/hip_runtime.h>

#include "device_utils.h"
#include "loong_internal.h"
#include "row_tiling.h"
#include "work_map.h"

namespace loong {
namespace {

constexpr float kRescaleSlack = 8.f;  // the running maximum may lag the true one by 2^8
constexpr int kFwdWaves = kRowWaves;

typedef __attribute__((address_space(3))) void lds_void_t;

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
  WorkMap map;     // units = batch x head groups, items = q tiles
};

template <int D, int KS>
struct FwdCfg {
  static constexpr int NT = kFwdWaves * 64;
  static constexpr int NRB = kFwdWaves / KS;       // 32-row blocks per workgroup
  static constexpr int BNS = KS == 1 ? 64 : 32;    // keys per wave and iteration
  static constexpr int TK = KS * BNS;              // keys staged per iteration
  static constexpr int ROWB = D * 2;               // bytes per K or V row
  static constexpr int CH = D / 8;                 // 16-byte pieces per row
  static constexpr int RP = 256 / ROWB;            // rows per 256 bytes (one sweep over all LDS banks)
  static constexpr int TILE_B = TK * ROWB;         // bytes of one K (or V) tile
  static constexpr int BUF_B = 2 * TILE_B;
  static constexpr int NBUF = BUF_B * 4 <= 131072 ? 4 : 2;
  static constexpr int PD = NBUF - 1;              // tiles in flight ahead of the one being used
  static constexpr int RPI = 1024 / ROWB;          // rows filled by one wave-level load
  static constexpr int KI = TILE_B / 1024 / kFwdWaves;  // loads per wave per K (or V) tile
  static constexpr int SLOT_F4 = (D / 32) * 4 + 1; // float4 per lane of one wave's partial result
  static constexpr int TILE_BYTES = NBUF * BUF_B;
  static constexpr int COMB_BYTES = (KS > 1 ? KS : 0) * NRB * SLOT_F4 * 64 * 16;
  static constexpr int SMEM_BYTES = TILE_BYTES > COMB_BYTES ? TILE_BYTES : COMB_BYTES;
  static_assert(KI >= 1 && KI * 1024 * kFwdWaves == TILE_B, "tile must split evenly over the waves");
};

template <class E, int D, int KS>
__global__ __launch_bounds__(kFwdWaves * 64) void fwd_kernel(const FwdParams p) {
  using C = FwdCfg<D, KS>;
  constexpr int NRB = C::NRB, BNS = C::BNS, TK = C::TK, NBUF = C::NBUF, PD = C::PD, KI = C::KI;
  constexpr int NJB = BNS / 32, NDB = D / 32, NKS = D / 16, ROWB = C::ROWB, CH = C::CH, RP = C::RP;
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

  float* out_row = p.out + b * p.os[0] + h * p.os[1] + (int64_t)my_row * p.os[2];
  float* lse_ptr = p.lse + ((int64_t)b * p.Hq + h) * p.q_len + my_row;

  if (total_t == 0) {  // nothing visible: neutral partial result, or leave the running one
    if (!p.fuse && ksp == 0 && row_ok) {
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq)
          *reinterpret_cast<float4*>(out_row + db * 32 + 8 * vq + 4 * hh) = make_float4(0.f, 0.f, 0.f, 0.f);
      if (hh == 0) *lse_ptr = -INFINITY;
    }
    return;
  }

  // ---- staging: global -> LDS directly.  Load i of this wave fills LDS bytes
  // [(wave + 8 i) * 1024, +1024) of the K (or V) tile: row (wave + 8 i) * RPI + lane / CH,
  // piece position lane % CH, which holds piece (position ^ swizzle(row)) of that row.
  const unsigned char* kbase = reinterpret_cast<const unsigned char*>(p.k + b * p.ks[0] + hk * p.ks[1]);
  const unsigned char* vbase = reinterpret_cast<const unsigned char*>(p.v + b * p.ks[0] + hk * p.ks[1]);
  const int64_t rowbytes = p.ks[2] * 2;
  const int ld_row = wave * C::RPI + lane / CH;  // row inside the tile for i = 0; later loads add 8*RPI rows
  const int ld_pos = lane % CH;
  const uint32_t k_piece = (uint32_t)(ld_pos ^ ((ld_row / RP) & (CH - 1))) * 16;
  const uint32_t v_piece = (uint32_t)(ld_pos ^ (((ld_row / RP) & (4 / RP - 1)) * 4)) * 16;
  const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_void_t*)smem;  // LDS byte address of the buffers
  auto tile_of = [&](int t, int& kb, int& j0) {
    kb = t < ntk0 ? 0 : 1;
    j0 = (t - (kb ? ntk0 : 0)) * TK;
  };
  // byte offsets of this lane's pieces from the first row of a tile (full tiles only; the
  // 32-bit form needs TK rows to span less than 4 GiB, else every tile takes the general path)
  const bool narrow = rowbytes * TK < (int64_t(1) << 32);
  uint32_t k_off[KI], v_off[KI];
#pragma unroll
  for (int i = 0; i < KI; ++i) {
    const uint32_t ro = (uint32_t)(ld_row + i * 8 * C::RPI) * (uint32_t)rowbytes;
    k_off[i] = ro + k_piece;
    v_off[i] = ro + v_piece;
  }
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
        load_to_lds_16(kbase + tb, k_off[i], kl + i * 8192);
        load_to_lds_16(vbase + tb, v_off[i], vl + i * 8192);
      }
    } else {
#pragma unroll
      for (int i = 0; i < KI; ++i) {
        const int r = min(ld_row + i * 8 * C::RPI, last);
        const int64_t ro = tb + (int64_t)r * rowbytes;
        load_to_lds_16(kbase + ro + k_piece, kl + i * 8192);
        load_to_lds_16(vbase + ro + v_piece, vl + i * 8192);
      }
    }
  };

  // ---- LDS read offsets of this lane (bytes inside a tile; the wave's split and the block
  // and slice indices are added as constants)
  // K operand: row l32 (+32 jb), pieces 2 ks + hh
  uint32_t k_rd[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) k_rd[ks] = l32 * ROWB + ((2 * ks + hh) ^ ((l32 / RP) & (CH - 1))) * 16;
  // V^T operand via transposing reads: in a group of 16 lanes, lane i points at row i / 4
  // of a run of four keys and at columns 4 (i % 4) .. +3 of a 16-column strip; it receives
  // the four keys of column i of the strip.  Lanes 0-31 / 32-63 take runs 4 hh .. 4 hh + 3.
  // The 32 lanes served in one clock cover four rows x four adjacent pieces (both strips):
  // the rows' XORs are four pieces apart.
  uint32_t v_rd[NDB];
  {
    const int i16 = lane & 15, r = i16 >> 2, qd = i16 & 3, strip = (lane >> 4) & 1;
    const int sw = ((r / RP) & (4 / RP - 1)) * 4;
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      const int piece = db * 4 + strip * 2 + (qd >> 1);
      v_rd[db] = (4 * hh + r) * ROWB + (piece ^ sw) * 16 + (qd & 1) * 8;
    }
  }

  // ---- per-tile pieces.  A wave skips a tile whose keys (its share of the staged tile) lie
  // past the end of the segment or past all of its rows.
  auto my_keys = [&](int t, int& j0, int& klen, bool& isdiag) {
    int kb;
    tile_of(t, kb, j0);
    j0 += ksp * BNS;
    klen = kb ? klen1 : klen0;
    isdiag = (kb ? cls1 : cls0) == LOONG_DIAG;
    return wave_live && j0 < klen && !(isdiag && j0 > wrow0 + 31);
  };

  // ---- pipeline: PD tiles in flight.  The first tiles are requested before the Q fragments
  // and the running state, so that the three latencies overlap; everything is then waited
  // for before the loop, so that no counter wait of the compiler's own ends up inside it,
  // where it would also wait for the tiles in flight.
#pragma unroll
  for (int t = 0; t < PD; ++t)
    if (t < total_t) issue_tile(t);

  // ---- Q fragments (B operand of S^T = K Q^T): row my_row, columns 16*ks + 8*hh .. +7
  bf16x8_t qf[NKS];
  {
    const uint16_t* qrow = p.q + b * p.qs[0] + h * p.qs[1] + (int64_t)my_row * p.qs[2];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(qrow + ks * 16 + hh * 8));
  }

  // ---- running state: maximum (log2 units), partial row sum of this half, O^T accumulators.
  // Only split 0 starts from the running result; its rows of `out` are requested together
  // with the LSE (one round trip to memory, not two) and dropped if the LSE says "empty".
  float m_run = -INFINITY, l_run = 0.f;
  floatx16_t o[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
  if (p.fuse && ksp == 0) {
    const float prev = *lse_ptr;
    float4 x[NDB][4];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) x[db][vq] = *reinterpret_cast<const float4*>(out_row + db * 32 + 8 * vq + 4 * hh);
    if (prev != -INFINITY) {
      m_run = prev * kLog2e;
      l_run = hh == 0 ? 1.f : 0.f;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          o[db][4 * vq + 0] = x[db][vq].x; o[db][4 * vq + 1] = x[db][vq].y;
          o[db][4 * vq + 2] = x[db][vq].z; o[db][4 * vq + 3] = x[db][vq].w;
        }
    }
  }

  wait_vmcnt<0>();
  const bool stage_late = PD == 1 && wave >= kFwdWaves / 2;  // waves w and w + 4 share a SIMD

  for (int t = 0; t < total_t; ++t) {
    // this wave's loads of tile t have landed when at most the later tiles' are outstanding
    const int later = min(PD - 1, total_t - 1 - t);
    if (later >= 2) wait_vmcnt<2 * 2 * KI>();
    else if (later == 1) wait_vmcnt<2 * KI>();
    else wait_vmcnt<0>();
    __syncthreads();  // every wave's part of tile t is in LDS; everyone has finished tile t-1
    // Tile t+PD goes into the buffer tile t-1 used.  A wave is held at each staging load
    // until the address unit has taken it (16 clocks per load, one unit per CU).  With a
    // single tile of look-ahead (the 64 KB tiles of four key splits) that hold is the largest
    // part of an iteration, and the two waves of a SIMD then stage at different times: one
    // right here, its partner behind its score product, each while the other computes
    // (3-5 % there; with deeper look-ahead staggering measured 7-10 % slower).
    const bool more = t + PD < total_t;
    if (more && !stage_late) issue_tile(t + PD);

    int j0, klen;
    bool isdiag;
    if (!my_keys(t, j0, klen, isdiag)) {
      if (more && stage_late) issue_tile(t + PD);
      continue;
    }
    const unsigned char* Kt = smem + (t % NBUF) * C::BUF_B + ksp * BNS * ROWB;
    const unsigned char* Vt = smem + (t % NBUF) * C::BUF_B + C::TILE_B + ksp * BNS * ROWB;

    // ---- S^T = K Q^T.  The K operands are requested PF products ahead (in program order, held
    // there by the scheduling barriers): left to itself the compiler keeps two reads in flight
    // and every pair of products then waits out a full LDS latency.
    floatx16_t s[NJB];
    {
      constexpr int NIT = NKS * NJB, PF = NIT >= 16 ? 6 : 4;
      auto k_frag = [&](int it) {
        return as_bf16x8(*reinterpret_cast<const uint4*>(Kt + (it % NJB) * 32 * ROWB + k_rd[it / NJB]));
      };
      bf16x8_t ring[PF + 1];
      static_for<0, PF>([&](auto i) { ring[i.value] = k_frag(i.value); });
      floatx16_t zero;
#pragma unroll
      for (int v = 0; v < 16; ++v) zero[v] = 0.f;
      static_for<0, NIT>([&](auto i) {
        constexpr int it = i.value;
        if constexpr (it + PF < NIT) ring[(it + PF) % (PF + 1)] = k_frag(it + PF);
        __builtin_amdgcn_sched_barrier(0);
        s[it % NJB] = E::mfma(ring[it % (PF + 1)], qf[it / NJB], it < NJB ? zero : s[it % NJB]);
      });
    }
    if (more && stage_late) issue_tile(t + PD);
    // ---- mask (diagonal or ragged end only)
    if (j0 + BNS > klen || (isdiag && j0 + BNS - 1 > wrow0)) {
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
    mx = max_with_other_half(mx);
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
        pk[jb][sl] = make_uint4(E::pack2(e[8 * sl + 0], e[8 * sl + 1]), E::pack2(e[8 * sl + 2], e[8 * sl + 3]),
                                E::pack2(e[8 * sl + 4], e[8 * sl + 5]), E::pack2(e[8 * sl + 6], e[8 * sl + 7]));
    }
    // ---- O^T += V^T P^T.  Element e of the B operand is key 16 sl + 8 (e / 4) + 4 hh + e % 4
    // of block jb: the A operand is the run starting at key 16 sl + 4 hh and the run 8 keys on.
#pragma unroll
    for (int jb = 0; jb < NJB; ++jb)
#pragma unroll
      for (int sl = 0; sl < 2; ++sl)
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          const unsigned char* vp = Vt + (jb * 32 + sl * 16) * ROWB + v_rd[db];
          o[db] = E::mfma(read_tr_pair(vp, vp + 8 * ROWB), as_bf16x8(pk[jb][sl]), o[db]);
        }
  }

  // ---- combine the key splits through LDS: every split parks (m, l, O^T); split j then
  // folds column block j (32 columns) of all splits, so the four waves share the work
  // (with fewer column blocks than splits the surplus waves leave).
  if (KS > 1) {
    __syncthreads();  // all reads of the last tile are done: the tile buffers are reused
    float4* slots = reinterpret_cast<float4*>(smem);
    {
      float4* mine = slots + (ksp * NRB + rb) * C::SLOT_F4 * 64 + lane;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq)
          mine[(db * 4 + vq) * 64] = make_float4(o[db][4 * vq], o[db][4 * vq + 1], o[db][4 * vq + 2], o[db][4 * vq + 3]);
      mine[(NDB * 4) * 64] = make_float4(m_run, l_run, 0.f, 0.f);
    }
    __syncthreads();
    constexpr int DBW = (NDB + KS - 1) / KS;  // column blocks per wave
    const int db0 = ksp * DBW;
    if (db0 >= NDB) return;
    // common maximum and the weights of the splits (fixed order: bit-reproducible)
    float m_all = -INFINITY;
    float ms[KS], ls[KS];
#pragma unroll
    for (int sp = 0; sp < KS; ++sp) {
      const float4 st = slots[((sp * NRB + rb) * C::SLOT_F4 + NDB * 4) * 64 + lane];
      ms[sp] = st.x; ls[sp] = st.y;
      m_all = fmaxf(m_all, st.x);
    }
    const float m_ref = m_all == -INFINITY ? 0.f : m_all;
    float l_all = 0.f, w[KS];
#pragma unroll
    for (int sp = 0; sp < KS; ++sp) {
      w[sp] = fast_exp2(ms[sp] - m_ref);  // exp2(-inf) = 0
      l_all += ls[sp] * w[sp];
    }
    const float l_tot = sum_with_other_half(l_all);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    if (row_ok) {
#pragma unroll
      for (int d2 = 0; d2 < DBW; ++d2) {
        const int db = db0 + d2;
        if (db >= NDB) break;
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
          for (int sp = 0; sp < KS; ++sp) {
            const float4 xv = slots[((sp * NRB + rb) * C::SLOT_F4 + db * 4 + vq) * 64 + lane];
            acc.x += xv.x * w[sp]; acc.y += xv.y * w[sp]; acc.z += xv.z * w[sp]; acc.w += xv.w * w[sp];
          }
          *reinterpret_cast<float4*>(out_row + db * 32 + 8 * vq + 4 * hh) =
              make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
        }
      }
      if (ksp == 0 && hh == 0) *lse_ptr = l_tot > 0.f ? (m_all + fast_log2(l_tot)) * kLn2 : -INFINITY;
    }
    return;
  }

  // ---- normalise and store
  const float l_tot = sum_with_other_half(l_run);
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

template <class E, int D, int KS>
int launch_cfg(FwdParams& p, hipStream_t st) {
  const RowTiling rt = make_row_tiling(p.g, p.G, p.Hq, p.B, kFwdWaves / KS, /*list_blind=*/!p.fuse);  // unfused: blind rows get the neutral result
  p.GS = rt.GS; p.ntile[0] = rt.ntile[0]; p.ntile[1] = rt.ntile[1];
  p.tiles_total = rt.tiles_total; p.hgroups = rt.hgroups;
  const int64_t total = rt.total_wg;
  if (total == 0) return LOONG_OK;
  if (total > 0x3ffffff0) return fail(LOONG_E_UNSUPPORTED, "forward grid too large");
  p.map = make_work_map((int64_t)p.B * rt.hgroups, rt.tiles_total);
  fwd_kernel<E, D, KS><<<dim3(p.map.grid), dim3(kFwdWaves * 64), 0, st>>>(p);
  return check_launch("loong_attn_step_fwd (bf16)");
}

template <class E>
int pick_cfg(FwdParams& p, int head_dim, int ks, hipStream_t st) {
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

int launch_fwd_bf16(const loong_step_desc& d, const StepGeom& g, const void* q, const void* k,
                    const void* v, float* out, float* lse, void* stream) {
  FwdParams p{};
  p.q = (const uint16_t*)q; p.k = (const uint16_t*)k; p.v = (const uint16_t*)v;
  p.out = out; p.lse = lse;
  p.B = d.batch; p.Hq = d.n_q_heads; p.Hkv = d.n_kv_heads; p.G = d.n_q_heads / d.n_kv_heads;
  for (int i = 0; i < 3; ++i) { p.qs[i] = d.q_stride[i]; p.ks[i] = d.kv_stride[i]; p.os[i] = d.o_stride[i]; }
  p.q_len = d.q_len; p.g = g; p.c = d.softmax_scale * kLog2e; p.fuse = (d.flags & LOONG_FUSE_MERGE) ? 1 : 0;
  hipStream_t st = static_cast<hipStream_t>(stream);
  DeviceFacts dev;
  if (int rc = device_facts(&dev)) return rc;
  const int ks = pick_key_splits(g, p.G, p.Hq, p.B, forced_key_splits(d.flags), dev.cus);
  if (d.dtype == LOONG_FP16) return pick_cfg<Fp16>(p, d.head_dim, ks, st);
  return pick_cfg<Bf16>(p, d.head_dim, ks, st);
}

}  // namespace loong
