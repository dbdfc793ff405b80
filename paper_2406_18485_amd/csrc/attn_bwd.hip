// Backward micro-step on the 16-bit matrix cores (element class E: bf16 or IEEE half; the text
// below says bf16 for both), dK/dV part: gradients of the visiting K/V chunk,
// recomputing the probabilities from the final softmax_lse (paper: Sec. 3.1 last paragraph;
// Sec. "Selective Checkpoint++").  This step's share of dQ comes from the row-owning pass
// in attn_bwd_dq.hip, launched right after this kernel.
//
// Work split.  A workgroup owns 128 keys of one kv head and walks over the 64-row query
// tiles of every q head of the group that can see them.  It has eight waves, two per SIMD:
// for each group of 32 keys a "P wave" and an "E wave" that sit on the same SIMD.
//   P wave   keeps the K rows (B operand) and the fp32 dV accumulator of its 32 keys:
//            S = Q K^T, P = exp2(S * scale * log2 e - LSE * log2 e), packed to bf16, handed
//            to its partner through LDS, then dV += P^T dO;
//   E wave   keeps the -V rows and the fp32 dK accumulator: T = delta - dO V^T straight out
//            of the matrix cores (the chain starts from C = delta), then E = P o T
//            (= -dS / scale), dK += E^T Q; dK is multiplied by -scale once, at the end.
// The E waves run one tile behind the P waves (P of tile t is consumed in the next iteration,
// from a double-buffered hand-over area; the query tiles stay in LDS for three iterations), so
// one workgroup barrier per tile suffices and neither role ever waits for the other.  The E
// waves, which have less element-wise work, also issue the staging loads.  A P wave's own
// dV += P^T dO of tile t also runs one iteration late, first thing after the barrier, from
// the P it kept in registers: the iteration then opens with matrix work on one wave of every
// SIMD while its partner issues the staging loads, instead of both starting with vector and
// memory instructions (2 % on the kernel, with the operand reads four matrix steps ahead).
// Splitting the roles halves the registers a wave must hold (so two waves fit a SIMD), and
// the two waves of a SIMD are in different kinds of work at any time: the vector issue port,
// which the matrix instructions share with the element-wise ones, is the unit that bounds
// this kernel, and every other instruction of one wave (LDS reads, waits, staging, scalar
// work) now hides behind the partner.
//
// Per query tile: Q, dO (row-major) and the rows' LSE and delta go from global memory
// straight into LDS, one tile ahead, with the 16-byte pieces of every row XOR-permuted so
// that both kinds of LDS read are free of bank conflicts: A operands of S / T are 16-byte
// reads of Q / dO rows (one key per lane, 16 query rows per 32x32 block in registers);
// the contractions over rows take P^T / E^T straight from registers as the A operand and
// transposing LDS reads of the same dO / Q tiles as the B operand.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>

#include "device_utils.h"
#include "loong_internal.h"
#include "work_map.h"

namespace loong {
namespace {

struct BwdParams {
  const uint16_t *q, *k, *v, *d_o;
  const float *lse, *delta;
  float *dk, *dv;
  int B, Hq, Hkv, G;
  int q_len, kv_len;
  int64_t qs[3], ks[3];
  StepGeom g;
  float scale, c;  // softmax scale; scale * log2(e)
  int accumulate;  // 1: the results are added to dk/dv instead of stored
  int nkt[2], kt_total;
  int nsplit;      // workgroups that share the query loop of one key tile
  uint32_t* ws_cnt;  // nsplit > 1: arrival counter per (batch, kv head, key tile), cleared before the launch
  float* ws_part;    // nsplit > 1: partial dK/dV of every (key tile, split), in accumulator layout
  WorkMap map;     // units = batch x kv heads, items = key tiles x splits
};

constexpr int kBwdWaves = 8;            // 4 key groups x {P wave, E wave}
constexpr int kBwdBN = 128;             // keys per workgroup
constexpr int kBwdBM = 64;              // query rows per iteration

template <int D>
struct BwdCfg {
  static constexpr int BM = kBwdBM, BN = kBwdBN;
  static constexpr int ROWB = D * 2;               // bytes per row of a Q / dO tile
  static constexpr int CH = D / 8;                 // 16-byte pieces per row
  static constexpr int RPI = 1024 / ROWB;          // rows filled by one wave-level load
  static constexpr int QT_B = BM * ROWB;           // bytes of a Q (or dO) tile
  static constexpr int LI = QT_B / 1024 / 4;       // loads per staging wave (the four E waves) per Q (or dO) tile
  static constexpr int STAGE_B = 2 * QT_B + 2 * BM * 4;  // Q, dO, lse, delta
  static constexpr int NSTAGE = 3;                 // tile being staged, tile of the P waves, tile of the E waves
  static constexpr int XCH_B = 4 * 2 * 2 * 1024;   // P hand-over: 4 key groups x 2 blocks x 2 halves x 64 lanes x 16 B
  static constexpr int SMEM_BYTES = NSTAGE * STAGE_B + 2 * XCH_B;
  static_assert(LI >= 1 && LI * 1024 * 4 == QT_B, "tile must split evenly over the staging waves");
};

template <class E, int D>
__global__ __launch_bounds__(kBwdWaves * 64) void bwd_dkv_kernel(const BwdParams p) {
  using C = BwdCfg<D>;
  constexpr int BM = C::BM, BN = C::BN, ROWB = C::ROWB, CH = C::CH, LI = C::LI;
  constexpr int NKS = D / 16, NDB = D / 32;
  static_assert(BM == 64, "the pipeline below is written for two 32-row blocks per tile");
  __shared__ __attribute__((aligned(1024))) unsigned char smem[C::SMEM_BYTES];

  // ---- which (batch, kv head, key tile, split)
  int bhk, rem;  // key tiles in storage order see ever fewer queries: that is the ranking
  if (!decode_work(p.map, blockIdx.x, bhk, rem)) return;
  const int kt = rem / p.nsplit, sp = rem - kt * p.nsplit;
  const int b = bhk / p.Hkv, hk = bhk - b * p.Hkv;
  const int kb = kt >= p.nkt[0] ? 1 : 0;
  const int koff0 = (kb ? kt - p.nkt[0] : kt) * BN;
  const Segment kseg = kb ? p.g.k[1] : p.g.k[0];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hh = lane >> 5;
  const int kg = wave & 3;           // key group: keys koff0 + 32 kg ..
  const bool p_wave = wave < 4;      // waves kg and kg + 4 share a SIMD
  const int my_koff = koff0 + 32 * kg + l32;
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
  // iteration -> (head of the group, tile inside the group's list); advanced without divisions
  struct Cursor { int gq, r; };
  auto advance = [&](Cursor& cu) {
    if (++cu.r == per_g) { cu.r = 0; ++cu.gq; }
  };
  auto decode = [&](const Cursor& cu, int& h, int& qa, int& i0) {
    qa = cu.r < cnt0 ? 0 : 1;
    i0 = (qa ? first1 + cu.r - cnt0 : first0 + cu.r) * BM;
    h = hk * p.G + cu.gq;
  };

  // ---- the wave's B operand: its K rows (P wave) or its V rows with the sign bits flipped
  // (E wave); row my_krow, columns 16 ks + 8 hh .. +7
  bf16x8_t bfrag[NKS];
  {
    const uint16_t* row = (p_wave ? p.k : p.v) + b * p.ks[0] + hk * p.ks[1] + my_krow * p.ks[2];
    const uint32_t flip = p_wave ? 0u : 0x80008000u;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      uint4 x = *reinterpret_cast<const uint4*>(row + ks * 16 + hh * 8);
      x.x ^= flip; x.y ^= flip; x.z ^= flip; x.w ^= flip;
      bfrag[ks] = as_bf16x8(x);
      // K comes with scale * log2 e folded in (rounded to 16 bits again): the score product then ends
      // in the exponent's units and its chains can start from the rows' offsets, which takes the
      // multiply-add per element off the vector port (4 % of the kernel).  The second rounding
      // changes P by less than rounding P itself to 16 bits does.
      if (p_wave) bfrag[ks] = scaled_fragment<E>(bfrag[ks], p.c);
    }
  }

  // ---- per-lane pieces of the staging and of the LDS reads
  const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;
  // direct loads (E waves): load i of staging wave kg fills LDS bytes [(kg + 4 i) * 1024, +1024) of a tile
  const int ld_row = kg * C::RPI + lane / CH;  // row inside the tile for i = 0; later loads add 4 * RPI rows
  const uint32_t ld_piece = (uint32_t)((lane % CH) ^ tile_swizzle<D>(ld_row)) * 16;
  const uint32_t q_rowbytes = (uint32_t)p.qs[2] * 2;  // validated: token stride < 2^24 elements
  uint32_t ld_off[LI];  // byte offset of this lane's piece from the tile's first row
#pragma unroll
  for (int i = 0; i < LI; ++i) ld_off[i] = (uint32_t)(ld_row + i * 4 * C::RPI) * q_rowbytes + ld_piece;
  // A operand of S / T: row l32 (+32 ib), pieces 2 ks + hh
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
  // P hand-over slot of this key group: [block][half of the block's 16 elements][lane] x 16 bytes
  unsigned char* const xch = smem + C::NSTAGE * C::STAGE_B + kg * 4096 + lane * 16;

  floatx16_t acc[NDB];  // dV (P wave) or dK / -scale (E wave) of the wave's 32 keys
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;

  // ---- staging of one query tile by the E waves: Q, dO rows and their LSE / delta, global -> LDS
  auto issue_tile = [&](const Cursor& cu, int stage) {
    if (p_wave) return;
    int h, qa, i0;
    decode(cu, h, qa, i0);
    const int qlen = qa ? qlen1 : qlen0, qstart = qa ? qstart1 : qstart0;
    const int last = qlen - 1 - i0;
    const uint32_t st = smem_base + stage * C::STAGE_B;
    const int64_t tile_off = b * p.qs[0] + h * p.qs[1] + (int64_t)(qstart + i0) * p.qs[2];
    const unsigned char* qb = reinterpret_cast<const unsigned char*>(p.q + tile_off);
    const unsigned char* ob = reinterpret_cast<const unsigned char*>(p.d_o + tile_off);
    if (last >= BM - 1) {
#pragma unroll
      for (int i = 0; i < LI; ++i) {
        load_to_lds_16(qb, ld_off[i], st + (kg + 4 * i) * 1024);
        load_to_lds_16(ob, ld_off[i], st + C::QT_B + (kg + 4 * i) * 1024);
      }
    } else {  // ragged end of a segment: rows past the last one repeat it
#pragma unroll
      for (int i = 0; i < LI; ++i) {
        const uint32_t off = (uint32_t)min(ld_row + i * 4 * C::RPI, last) * q_rowbytes + ld_piece;
        load_to_lds_16(qb, off, st + (kg + 4 * i) * 1024);
        load_to_lds_16(ob, off, st + C::QT_B + (kg + 4 * i) * 1024);
      }
    }
    if (kg < 2) {  // E wave 0: the 64 rows' LSE, E wave 1: their delta
      const int64_t row = ((int64_t)b * p.Hq + h) * p.q_len + qstart + i0 + min(lane, last);
      load_to_lds_4((kg ? p.delta : p.lse) + row, st + 2 * C::QT_B + kg * BM * 4);
    }
  };

  Cursor cur, nxt;
  cur.gq = it_begin / max(per_g, 1);
  cur.r = it_begin - cur.gq * per_g;
  nxt = cur;

  wait_vmcnt<0>();  // the K / V fragments are in: no counter wait of the compiler's lands in the loop
  if (it_begin < it_end) issue_tile(cur, 0);
  wait_vmcnt<0>();

  // P and E = P o T packed, two bf16 per word (elements 2 w, 2 w + 1 of block ib).  A P wave keeps
  // its P across the barrier: dV += P^T dO of tile t runs at the top of iteration t + 1.
  uint32_t w2[2][8];
  constexpr int PF = 4;  // LDS operands are requested PF matrix steps ahead
  // Iteration j: the P waves work on tile j, the E waves on tile j - 1, tile j + 1 is staged.
  int st_p = 0, st_e = 2, st_n = 1;  // LDS stages of those three tiles
  for (int it = it_begin; it <= it_end && it_begin < it_end; ++it) {
    __syncthreads();  // tile `it` is in LDS, P of tile it - 1 is handed over, tile it - 2 is finished with
    if (it + 1 < it_end) {
      advance(nxt);
      issue_tile(nxt, st_n);
    }
    const bool p_active = p_wave && it < it_end, e_active = !p_wave && it > it_begin;
    int h, qa, i0;
    decode(cur, h, qa, i0);
    const int qlen = qa ? qlen1 : qlen0;
    const bool isdiag = (qa ? clsq1 : clsq0) == LOONG_DIAG;
    const bool need_mask = i0 + BM > qlen || koff0 + BN > kseg.len || (isdiag && i0 < koff0 + BN - 1);
    const unsigned char* Qt = smem + (p_wave ? st_p : st_e) * C::STAGE_B;
    const unsigned char* Ot = Qt + C::QT_B;
    const float* lse_s = reinterpret_cast<const float*>(Qt + 2 * C::QT_B);
    const float* dl_s = lse_s + BM;
    unsigned char* const xch_w = xch + ((it - it_begin) & 1) * C::XCH_B;        // P of tile `it`
    const unsigned char* const xch_r = xch + ((it - it_begin + 1) & 1) * C::XCH_B;  // P of tile it - 1

    // Block ib = rows 32 ib .. 32 ib + 31 of the tile; register v of an accumulator is row
    // acc_row(v, hh) of the block.
    floatx16_t st2[2];
    // 2 NKS matrix steps of S (P wave: Q rows, K fragments) or T (E wave: dO rows, -V fragments)
    // of both blocks, block 1 after block 0; `between(k)` is called after step k.
    auto rows_product = [&](const unsigned char* tile, auto&& between) {
      auto operand = [&](int k) {
        return as_bf16x8(*reinterpret_cast<const uint4*>(tile + (k / NKS) * 32 * ROWB + row_rd[k % NKS]));
      };
      bf16x8_t ring[PF + 1];
      static_for<0, PF>([&](auto kc) { ring[kc.value] = operand(kc.value); });
      // An E wave runs its matrix steps at raised priority: its path from barrier to barrier is the
      // longer one, and with equal priorities the partner's vector instructions get between its
      // matrix instructions (1.5 % on the kernel; raising the P waves too, or instead: nothing)
      if (!p_wave) __builtin_amdgcn_s_setprio(3);
      static_for<0, 2 * NKS>([&](auto kc) {
        constexpr int k = decltype(kc)::value, ib = k / NKS, ks = k % NKS;
        if constexpr (k + PF < 2 * NKS) ring[(k + PF) % (PF + 1)] = operand(k + PF);
        st2[ib] = E::mfma(ring[k % (PF + 1)], bfrag[ks], st2[ib]);  // the chains start from the exponent offsets (P) or delta (E)
        between(kc);
        __builtin_amdgcn_sched_barrier(0);  // keep the operand reads ahead of their use
      });
      if (!p_wave) __builtin_amdgcn_s_setprio(0);
    };
    // 4 NDB matrix steps of acc += W^T X over the tile's 64 rows (W = pw or ew, X = dO or Q tile).
    // Element e of the A operand is row 16 sl + 8 (e / 4) + 4 hh + e % 4 of its block, so the
    // B operand is the run of four rows starting at 16 sl + 4 hh and the run 8 rows on.
    auto cols_product = [&](const unsigned char* tile, auto&& before) {
      auto operand = [&](int k) {
        const int ib = k / (2 * NDB), sl = (k / NDB) % 2, db = k % NDB;
        const unsigned char* base = tile + (ib * 32 + sl * 16) * ROWB;
        return read_tr_pair(base + tr_lo[db], base + tr_hi[db]);
      };
      bf16x8_t ring[PF + 1];
      static_for<0, PF>([&](auto kc) { ring[kc.value] = operand(kc.value); });
      if (!p_wave) __builtin_amdgcn_s_setprio(3);
      static_for<0, 4 * NDB>([&](auto kc) {
        constexpr int k = decltype(kc)::value, ib = k / (2 * NDB), sl = (k / NDB) % 2, db = k % NDB;
        if constexpr (k + PF < 4 * NDB) ring[(k + PF) % (PF + 1)] = operand(k + PF);
        before(kc);
        const bf16x8_t a = as_bf16x8(make_uint4(w2[ib][4 * sl], w2[ib][4 * sl + 1], w2[ib][4 * sl + 2], w2[ib][4 * sl + 3]));
        acc[db] = E::mfma(a, ring[k % (PF + 1)], acc[db]);
        __builtin_amdgcn_sched_barrier(0);
      });
      if (!p_wave) __builtin_amdgcn_s_setprio(0);
    };

    // dV += P^T dO of tile it - 1 (its dO is still staged: the E waves work on that tile now)
    if (p_wave && it > it_begin) cols_product(smem + st_e * C::STAGE_B + C::QT_B, [](auto) {});
    if (p_active) {
      // exponent offsets -LSE log2 e, where the score chains start; masked pairs get -inf: P = 0
      // whatever the score
      floatx16_t (&nl)[2] = st2;
#pragma unroll
      for (int ib = 0; ib < 2; ++ib)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          const float4 L = *reinterpret_cast<const float4*>(&lse_s[ib * 32 + 8 * vq + 4 * hh]);
          nl[ib][4 * vq + 0] = L.x * -kLog2e; nl[ib][4 * vq + 1] = L.y * -kLog2e;
          nl[ib][4 * vq + 2] = L.z * -kLog2e; nl[ib][4 * vq + 3] = L.w * -kLog2e;
        }
      // a row whose LSE is -inf saw no key in the whole attention: its offset came out as +inf
      // and must be -inf (P = 0).  One look at the tile's 64 staged values per wave finds the case.
      const bool blind_row = __builtin_amdgcn_ballot_w64(lse_s[lane] == -INFINITY) != 0;
      if (need_mask || blind_row) {
#pragma unroll
        for (int ib = 0; ib < 2; ++ib)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int i_off = i0 + ib * 32 + acc_row(v, hh);
            const bool ok = key_ok && i_off < qlen && (!isdiag || my_koff <= i_off) && nl[ib][v] < INFINITY;
            nl[ib][v] = ok ? nl[ib][v] : -INFINITY;
          }
      }
      auto exps = [&](int ib, int w) {  // elements 2 w, 2 w + 1 of block ib
        const float p0 = fast_exp2(st2[ib][2 * w]);
        const float p1 = fast_exp2(st2[ib][2 * w + 1]);
        w2[ib][w] = E::pack2(p0, p1);
      };
      // S of both blocks; the exponentials of block 0 between the matrix steps of block 1
      rows_product(Qt, [&](auto kc) {
        constexpr int k = decltype(kc)::value;
        if constexpr (k >= NKS) static_for<0, 8 / NKS>([&](auto uc) { exps(0, (k - NKS) * (8 / NKS) + uc.value); });
      });
#pragma unroll
      for (int w = 0; w < 8; ++w) exps(1, w);
      // hand P to the partner wave
#pragma unroll
      for (int ib = 0; ib < 2; ++ib)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
          *reinterpret_cast<uint4*>(xch_w + (ib * 2 + hf) * 1024) =
              make_uint4(w2[ib][4 * hf], w2[ib][4 * hf + 1], w2[ib][4 * hf + 2], w2[ib][4 * hf + 3]);
    } else if (e_active) {
      // T = delta - dO V^T: the chains start from the rows' delta
#pragma unroll
      for (int ib = 0; ib < 2; ++ib)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          const float4 Dl = *reinterpret_cast<const float4*>(&dl_s[ib * 32 + 8 * vq + 4 * hh]);
          st2[ib][4 * vq + 0] = Dl.x; st2[ib][4 * vq + 1] = Dl.y; st2[ib][4 * vq + 2] = Dl.z; st2[ib][4 * vq + 3] = Dl.w;
        }
      rows_product(Ot, [](auto) {});
      uint32_t pw[2][8];
#pragma unroll
      for (int ib = 0; ib < 2; ++ib)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          const uint4 x = *reinterpret_cast<const uint4*>(xch_r + (ib * 2 + hf) * 1024);
          pw[ib][4 * hf] = x.x; pw[ib][4 * hf + 1] = x.y; pw[ib][4 * hf + 2] = x.z; pw[ib][4 * hf + 3] = x.w;
        }
      auto etimes = [&](int ib, int w) {  // E = P o T for elements 2 w, 2 w + 1 of block ib
        w2[ib][w] = E::pack2(E::lo(pw[ib][w]) * st2[ib][2 * w], E::hi(pw[ib][w]) * st2[ib][2 * w + 1]);
      };
#pragma unroll
      for (int w = 0; w < 8; ++w) etimes(0, w);
      // dK += E^T Q; the products of block 1 between the matrix steps of block 0
      cols_product(Qt, [&](auto kc) {
        constexpr int k = decltype(kc)::value;
        if constexpr (k < 2 * NDB) static_for<0, 8 / (2 * NDB)>([&](auto uc) { etimes(1, k * (8 / (2 * NDB)) + uc.value); });
      });
    }
    wait_vmcnt<0>();  // this wave's part of the next tile, issued a whole iteration ago
    if (it < it_end) advance(cur);
    const int freed = st_e;
    st_e = st_p; st_p = st_n; st_n = freed;
  }

  // ---- several workgroups shared this key tile's query loop: each parks its partial sums
  // in the caller's workspace, and the one that arrives last adds them up in split order,
  // so the result does not depend on the order of arrival (no atomics on dK/dV).
  // The partials cross between XCDs, whose L2s are not coherent for ordinary accesses.  A
  // device-scope fence would do (release: write back the XCD's L2, acquire: invalidate it),
  // but every workgroup would pay for the whole cache (measured: 1.4-1.8x the step time).
  // Instead every partial word is stored and loaded as a relaxed device-scope atomic, i.e.
  // written through to and read from the level all XCDs share; the stores are waited for
  // (vmcnt) before the workgroup's arrival is counted, and the last workgroup's loads are
  // issued after its count has returned.
  if (p.nsplit > 1) {
    __shared__ int s_last;
    const int tile_id = bhk * p.kt_total + kt;
    constexpr int WAVE_F = NDB * 16 * 64;  // floats per wave and slot
    float* parts = p.ws_part + (int64_t)tile_id * p.nsplit * (kBwdWaves * WAVE_F) + wave * WAVE_F + lane;
    {
      float* mine = parts + (int64_t)sp * (kBwdWaves * WAVE_F);
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          __hip_atomic_store(mine + (db * 16 + v) * 64, acc[db][v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    wait_vmcnt<0>();
    __syncthreads();
    if (tid == 0) {
      const uint32_t before = __hip_atomic_fetch_add(p.ws_cnt + tile_id, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_last = before == (uint32_t)p.nsplit - 1;
    }
    __syncthreads();
    if (!s_last) return;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;
    for (int s2 = 0; s2 < p.nsplit; ++s2) {
      const float* theirs = parts + (int64_t)s2 * (kBwdWaves * WAVE_F);
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          acc[db][v] += __hip_atomic_load(theirs + (db * 16 + v) * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }

  // ---- dV (P waves) and dK = -scale * (accumulated E^T Q) (E waves) of the wave's 32 keys.
  // A lane owns one column per block and 16 key rows; registers 4 vq .. 4 vq + 3 are four
  // consecutive keys.  Each such group is transposed across the four lanes of a quad (four
  // adjacent columns), so that a lane then holds four adjacent columns of one key and stores
  // 16 bytes: a quarter of the store instructions, which the address unit takes at the same
  // rate whatever their width (stored one float at a time, this epilogue took 3.2 us of a
  // 74 us launch).  This workgroup is the only one that writes these rows in this launch, so
  // accumulation is a plain read-modify-write.
  float* base = (p_wave ? p.dv : p.dk) + (((int64_t)b * p.Hkv + hk) * p.kv_len + kseg.start) * D;
  const float f = p_wave ? 1.f : -p.scale;
  const bool odd = lane & 1, upper = lane & 2;
  const int col4 = (l32 >> 2) * 4, key_in_group = l32 & 3;
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      const float r0 = acc[db][4 * vq] * f, r1 = acc[db][4 * vq + 1] * f, r2 = acc[db][4 * vq + 2] * f, r3 = acc[db][4 * vq + 3] * f;
      // lanes one apart exchange (r0, r1) and (r2, r3), then lanes two apart exchange the pairs
      // (every exchange runs in all lanes: a lane reads its partner's register, so none may sit in a branch)
      const float p0 = quad_swap1(r0), p1 = quad_swap1(r1), p2 = quad_swap1(r2), p3 = quad_swap1(r3);
      const float a0 = odd ? p1 : r0, a1 = odd ? r1 : p0, a2 = odd ? p3 : r2, a3 = odd ? r3 : p2;
      const float q0 = quad_swap2(a0), q1 = quad_swap2(a1), q2 = quad_swap2(a2), q3 = quad_swap2(a3);
      float4 x;
      x.x = upper ? q2 : a0; x.y = upper ? q3 : a1; x.z = upper ? a2 : q0; x.w = upper ? a3 : q1;
      const int koff = koff0 + 32 * kg + 8 * vq + 4 * hh + key_in_group;
      if (koff < kseg.len) {
        float4* dst = reinterpret_cast<float4*>(base + (int64_t)koff * D + db * 32 + col4);
        if (p.accumulate) {
          const float4 y = *dst;
          x.x += y.x; x.y += y.y; x.z += y.z; x.w += y.w;
        }
        *dst = x;
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

// The arrival counters a launch with shared query loops uses start from zero: cleared on the
// caller's stream right before it (a fill kernel, so the call can be captured in a graph).
__global__ __launch_bounds__(256) void clear_counters_kernel(int n, uint32_t* cnt) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) cnt[i] = 0u;
}

// Work list of a step: key tiles per key segment (only segments some query can see), whether
// a key segment nobody sees exists (its gradients are cleared by the zero pass), and how many
// workgroups share the query loop of a key tile: more than one when the listed tiles are
// fewer than the compute units (`cus`), and twice as many when a diagonal block makes the loop
// lengths uneven.
struct SplitPlan {
  int nkt[2], kt_total, nsplit;
  bool unseen_keys;
  int64_t busy;  // listed key tiles x kv heads x batch
};

SplitPlan plan_split(const StepGeom& g, int G, int Hkv, int B, int q_len, int cus) {
  constexpr int BM = kBwdBM, BN = kBwdBN;
  SplitPlan s{};
  bool diag = false;
  for (int kb = 0; kb < 2; ++kb) {
    bool seen = false;
    if (kb < g.nk)
      for (int a = 0; a < g.nq; ++a) {
        seen |= g.cls[a][kb] != LOONG_SKIP && g.q[a].len > 0;
        diag |= g.cls[a][kb] == LOONG_DIAG;
      }
    s.nkt[kb] = seen ? (g.k[kb].len + BN - 1) / BN : 0;
    s.kt_total += s.nkt[kb];
    s.unseen_keys |= kb < g.nk && !seen && g.k[kb].len > 0;
  }
  s.busy = (int64_t)s.kt_total * Hkv * B;
  int nsplit = 1;
  const int64_t q_tiles = std::max<int64_t>((int64_t)G * ((q_len + BM - 1) / BM), 1);
  if (s.busy > 0 && s.busy < cus) nsplit = (int)std::min<int64_t>((cus + s.busy - 1) / s.busy, 16);
  if (diag && s.busy * nsplit <= 2 * cus) nsplit *= 2;
  // The last workgroup of a key tile adds up all its partial sums alone, at one CU's memory
  // rate (about 1.1 us per split), while a split shortens the loop by q_tiles x 1.9 us / n:
  // past n = sqrt(1.76 q_tiles) more splits lengthen the launch.
  nsplit = (int)std::min<int64_t>(nsplit, std::max<int64_t>(2, (int64_t)std::sqrt(1.76 * (double)q_tiles)));
  nsplit = (int)std::min<int64_t>(nsplit, q_tiles);
  if (s.busy > kWsCounters) nsplit = 1;  // (cannot happen: loops are only shared when key tiles are few)
  s.nsplit = nsplit;
  return s;
}

// bytes of partial sums one launch parks in the workspace
size_t partial_bytes(const SplitPlan& s, int head_dim) {
  return s.nsplit > 1 ? (size_t)s.busy * s.nsplit * kBwdWaves * (head_dim / 32) * 16 * 64 * sizeof(float) : 0;
}

template <class E, int D>
int launch_d(BwdParams& p, bool accumulate, void* workspace, int64_t workspace_bytes, hipStream_t st) {
  // Only key tiles that some query can see are listed (eight equal ranges of the list, one
  // per XCD, then carry equal work).
  const SplitPlan plan = plan_split(p.g, p.G, p.Hkv, p.B, p.q_len, planning_cus());
  p.nkt[0] = plan.nkt[0]; p.nkt[1] = plan.nkt[1]; p.kt_total = plan.kt_total;
  const bool unseen_keys = plan.unseen_keys;
  const int64_t base = plan.busy;
  const int nsplit = plan.nsplit;
  p.nsplit = nsplit;
  p.accumulate = accumulate ? 1 : 0;
  const int64_t total = base * nsplit;
  if (total > 0x3ffffff0) return fail(LOONG_E_UNSUPPORTED, "backward grid too large");
  p.map = make_work_map((int64_t)p.Hkv * p.B, (int64_t)p.kt_total * nsplit);
  if (nsplit > 1) {  // (size and alignment were checked by the entry point, against the same plan)
    if (!workspace || workspace_bytes < kWsHeadBytes + (int64_t)partial_bytes(plan, D))
      return fail(LOONG_E_SHAPE, "loong_attn_step_bwd: workspace too small");
    p.ws_cnt = static_cast<uint32_t*>(workspace);
    p.ws_part = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + kWsHeadBytes);
  }
  DeviceFacts dev;
  if (int rc = device_facts(&dev)) return rc;
  if (unseen_keys && !accumulate) {
    const int64_t n4 = (int64_t)p.B * p.Hkv * p.kv_len * D / 4;
    zero_kernel<<<dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st>>>(n4, reinterpret_cast<float4*>(p.dk),
                                                                          reinterpret_cast<float4*>(p.dv));
    if (int rc = check_launch("loong_attn_step_bwd (clear dk/dv)")) return rc;
  }
  if (total == 0) return LOONG_OK;
  if (nsplit > 1) {
    clear_counters_kernel<<<dim3((unsigned)((base + 255) / 256)), dim3(256), 0, st>>>((int)base, p.ws_cnt);
    if (int rc = check_launch("loong_attn_step_bwd (clear counters)")) return rc;
  }
  bwd_dkv_kernel<E, D><<<dim3(p.map.grid), dim3(kBwdWaves * 64), 0, st>>>(p);
  return check_launch("loong_attn_step_bwd (bf16, dK/dV)");
}

}  // namespace

int launch_bwd_bf16(const loong_step_desc& d, const StepGeom& g, const void* q, const void* k,
                    const void* v, const void* d_o, const float* lse, const float* delta, float* dq,
                    float* dk, float* dv, void* workspace, int64_t workspace_bytes, void* stream) {
  if (d.kv_len == 0) return LOONG_OK;
  BwdParams p{};
  p.q = (const uint16_t*)q; p.k = (const uint16_t*)k; p.v = (const uint16_t*)v; p.d_o = (const uint16_t*)d_o;
  p.lse = lse; p.delta = delta; p.dk = dk; p.dv = dv;
  p.B = d.batch; p.Hq = d.n_q_heads; p.Hkv = d.n_kv_heads; p.G = d.n_q_heads / d.n_kv_heads;
  p.q_len = d.q_len; p.kv_len = d.kv_len;
  for (int i = 0; i < 3; ++i) { p.qs[i] = d.q_stride[i]; p.ks[i] = d.kv_stride[i]; }
  p.g = g; p.scale = d.softmax_scale; p.c = d.softmax_scale * kLog2e;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool accumulate = d.flags & LOONG_ACCUM_DKV;
  if (!(d.flags & LOONG_BWD_ONLY_DQ)) {
    const int rc = d.dtype == LOONG_FP16
                       ? (d.head_dim == 128 ? launch_d<Fp16, 128>(p, accumulate, workspace, workspace_bytes, st)
                                            : launch_d<Fp16, 64>(p, accumulate, workspace, workspace_bytes, st))
                       : (d.head_dim == 128 ? launch_d<Bf16, 128>(p, accumulate, workspace, workspace_bytes, st)
                                            : launch_d<Bf16, 64>(p, accumulate, workspace, workspace_bytes, st));
    if (rc != LOONG_OK) return rc;
  }
  if (d.flags & LOONG_BWD_ONLY_DKV) return LOONG_OK;
  return launch_bwd_dq_bf16(d, g, q, k, v, d_o, lse, delta, dq, stream);
}

int64_t bwd_workspace_bytes_bf16(const loong_step_desc& d, const StepGeom& g) {
  if (d.kv_len == 0 || d.batch == 0 || (d.flags & LOONG_BWD_ONLY_DQ)) return 0;
  const SplitPlan plan = plan_split(g, d.n_q_heads / d.n_kv_heads, d.n_kv_heads, d.batch, d.q_len, planning_cus());
  return plan.nsplit > 1 ? kWsHeadBytes + (int64_t)partial_bytes(plan, d.head_dim) : 0;
}

}  // namespace loong
