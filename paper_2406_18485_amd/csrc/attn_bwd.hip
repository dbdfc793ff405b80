// Backward micro-step on bf16 matrix cores, dK/dV part: gradients of the visiting K/V chunk,
// recomputing the probabilities from the final softmax_lse (paper: Sec. 3.1 last paragraph;
// Sec. "Selective Checkpoint++").  This step's share of dQ comes from the row-owning pass
// in attn_bwd_dq.hip, launched right after this kernel.
//
// Work split.  A workgroup of 4 waves (one per SIMD, up to 512 registers each) owns 128 keys
// of one kv head, 32 per wave, and walks over the 64-row query tiles of every q head of
// the group that can see them.  Loop-invariant in registers: the wave's K and V rows as B
// operands of S = Q K^T and dP = dO V^T (V negated, see below) and the fp32 dK / dV
// accumulators.
//
// Per query tile: Q, dO (row-major) and the rows' LSE and delta go from global memory
// straight into LDS, one tile ahead, with the 16-byte pieces of every row XOR-permuted so
// that both kinds of LDS read below are free of bank conflicts.
//   S, T      A operand = 16-byte reads of Q / dO rows; accumulators put one key per lane
//             and 16 query rows per 32x32 block in registers.  T = delta - dP comes out of
//             the matrix cores directly: the chain starts from C = delta and multiplies
//             by -V;
//   P         exp2(S * scale * log2 e - LSE * log2 e);  E = P o T = -dS / scale;
//   dV, dK    contraction over rows: A operand = P^T / E^T straight from those
//             accumulators (packed to bf16), B operand = transposing LDS reads of the same
//             dO / Q tiles; dK is multiplied by -scale once, at the end.
// The tile's two 32-row blocks are software-pipelined: the element-wise work on one block is
// written between the matrix instructions of the other, so both units stay busy although a
// SIMD holds a single wave.
#include <hip/hip_runtime.h>

#include <algorithm>

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
  int add_dkv;     // 1: dk/dv are added to with atomics (accumulate flag or split iteration space)
  int nkt[2], kt_total;
  int nsplit;
  WorkMap map;     // units = batch x kv heads, items = key tiles x splits
};

constexpr int kBwdWaves = 4;
constexpr int kBwdBN = 32 * kBwdWaves;  // keys per workgroup
constexpr int kBwdBM = 64;              // query rows per iteration

template <int D>
struct BwdCfg {
  static constexpr int BM = kBwdBM, BN = kBwdBN;
  static constexpr int ROWB = D * 2;               // bytes per row of a Q / dO tile
  static constexpr int CH = D / 8;                 // 16-byte pieces per row
  static constexpr int RPI = 1024 / ROWB;          // rows filled by one wave-level load
  static constexpr int QT_B = BM * ROWB;           // bytes of a Q (or dO) tile
  static constexpr int LI = QT_B / 1024 / kBwdWaves;  // loads per wave per Q (or dO) tile
  static constexpr int STAGE_B = 2 * QT_B + 2 * BM * 4;  // Q, dO, lse, delta
  static constexpr int SMEM_BYTES = 2 * STAGE_B;
};

template <int D>
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

  // ---- K and V rows of this wave as B operands (row my_krow, columns 16 ks + 8 hh .. +7);
  // V with the sign bits flipped
  bf16x8_t kf[NKS], vfn[NKS];
  {
    const uint16_t* krow = p.k + b * p.ks[0] + hk * p.ks[1] + my_krow * p.ks[2];
    const uint16_t* vrow = p.v + b * p.ks[0] + hk * p.ks[1] + my_krow * p.ks[2];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      kf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(krow + ks * 16 + hh * 8));
      uint4 x = *reinterpret_cast<const uint4*>(vrow + ks * 16 + hh * 8);
      x.x ^= 0x80008000u; x.y ^= 0x80008000u; x.z ^= 0x80008000u; x.w ^= 0x80008000u;
      vfn[ks] = as_bf16x8(x);
    }
  }

  // ---- per-lane pieces of the staging and of the LDS reads
  const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;
  // direct loads: load i of this wave fills LDS bytes [(wave + 4 i) * 1024, +1024) of a tile
  const int ld_row = wave * C::RPI + lane / CH;  // row inside the tile for i = 0; later loads add 4 * RPI rows
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

  floatx16_t dk[NDB], dv[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dk[db][v] = 0.f; dv[db][v] = 0.f; }

  // ---- staging of one query tile: Q, dO rows and their LSE / delta, global -> LDS
  auto issue_tile = [&](const Cursor& cu, int stage) {
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
        load_to_lds_16(qb, ld_off[i], st + (wave + 4 * i) * 1024);
        load_to_lds_16(ob, ld_off[i], st + C::QT_B + (wave + 4 * i) * 1024);
      }
    } else {  // ragged end of a segment: rows past the last one repeat it
#pragma unroll
      for (int i = 0; i < LI; ++i) {
        const uint32_t off = (uint32_t)min(ld_row + i * 4 * C::RPI, last) * q_rowbytes + ld_piece;
        load_to_lds_16(qb, off, st + (wave + 4 * i) * 1024);
        load_to_lds_16(ob, off, st + C::QT_B + (wave + 4 * i) * 1024);
      }
    }
    if (wave < 2) {  // wave 0: the 64 rows' LSE, wave 1: their delta
      const int64_t row = ((int64_t)b * p.Hq + h) * p.q_len + qstart + i0 + min(lane, last);
      load_to_lds_4((wave ? p.delta : p.lse) + row, st + 2 * C::QT_B + wave * BM * 4);
    }
  };

  Cursor cur, nxt;
  cur.gq = it_begin / max(per_g, 1);
  cur.r = it_begin - cur.gq * per_g;
  nxt = cur;

  wait_vmcnt<0>();  // K / V fragments are in: no counter wait of the compiler's lands in the loop
  if (it_begin < it_end) issue_tile(cur, 0);
  wait_vmcnt<0>();

  int stage = 0;
  for (int it = it_begin; it < it_end; ++it, stage ^= 1, advance(cur)) {
    // the accumulators live in the accumulation registers for the whole loop (a hint: nothing
    // is emitted here, but the register allocator may not park them among the vector registers)
#pragma unroll
    for (int db = 0; db < NDB; ++db) asm volatile("" : "+a"(dk[db]), "+a"(dv[db]));
    __syncthreads();  // tile `it` is in LDS (each wave waited for its part); iteration it - 1 is finished
    if (it + 1 < it_end) {
      advance(nxt);
      issue_tile(nxt, stage ^ 1);
    }
    int h, qa, i0;
    decode(cur, h, qa, i0);
    const int qlen = qa ? qlen1 : qlen0;
    const bool isdiag = (qa ? clsq1 : clsq0) == LOONG_DIAG;
    const bool need_mask = i0 + BM > qlen || koff0 + BN > kseg.len || (isdiag && i0 < koff0 + BN - 1);
    const unsigned char* Qt = smem + stage * C::STAGE_B;
    const unsigned char* Ot = Qt + C::QT_B;
    const float* lse_s = reinterpret_cast<const float*>(Qt + 2 * C::QT_B);
    const float* dl_s = lse_s + BM;

    // One tile.  Block ib = rows 32 ib .. 32 ib + 31; register v of an accumulator is row
    // acc_row(v, hh) of the block.  The tile is a sequence of 4 NS matrix steps: S and T of
    // block 0 (alternating), of block 1, then dV and dK with block 0, with block 1; the
    // LDS operands are requested a batch of PF steps ahead (one counter wait per batch), and
    // the element-wise work on block 0 (1) is spread over the steps of the second (third)
    // quarter.
    constexpr int NS = 2 * NKS;    // matrix steps per quarter (== 4 * NDB)
    constexpr int EPS = 16 / NS;   // elements per matrix step
    constexpr int PF = 4;          // operands are read in batches of PF, one batch ahead of their use
    static_assert(NS == 4 * NDB && EPS * NS == 16, "quarters of equal length");
    floatx16_t s[2], t[2];
    float nl[2][16];
    uint32_t pw[2][8], ew[2][8];  // P and E = P o T, two bf16 per word: elements 2 w, 2 w + 1
    // C operand of the T chains (the rows' delta) and exponent offsets -LSE log2 e
#pragma unroll
    for (int ib = 0; ib < 2; ++ib)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        const float4 L = *reinterpret_cast<const float4*>(&lse_s[ib * 32 + 8 * vq + 4 * hh]);
        const float4 Dl = *reinterpret_cast<const float4*>(&dl_s[ib * 32 + 8 * vq + 4 * hh]);
        nl[ib][4 * vq + 0] = L.x * -kLog2e; nl[ib][4 * vq + 1] = L.y * -kLog2e;
        nl[ib][4 * vq + 2] = L.z * -kLog2e; nl[ib][4 * vq + 3] = L.w * -kLog2e;
        t[ib][4 * vq + 0] = Dl.x; t[ib][4 * vq + 1] = Dl.y; t[ib][4 * vq + 2] = Dl.z; t[ib][4 * vq + 3] = Dl.w;
      }
    if (need_mask) {  // masked pairs get the exponent offset -inf: P = 0 whatever the score
#pragma unroll
      for (int ib = 0; ib < 2; ++ib)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int i_off = i0 + ib * 32 + acc_row(v, hh);
          const bool ok = key_ok && i_off < qlen && (!isdiag || my_koff <= i_off);
          nl[ib][v] = ok ? nl[ib][v] : -INFINITY;
        }
    }
    // LDS operand of matrix step k: a 16-byte piece of a Q / dO row, or two transposing reads
    // (element e of the A operand of dV / dK is row 16 sl + 8 (e / 4) + 4 hh + e % 4 of its
    // block, so the B operand is the run of four rows starting at 16 sl + 4 hh and the run
    // 8 rows on)
    auto operand = [&](int k) -> bf16x8_t {
      const int quarter = k / NS, j = k % NS, second = j & 1;
      if (quarter < 2)
        return as_bf16x8(*reinterpret_cast<const uint4*>((second ? Ot : Qt) + quarter * 32 * ROWB + row_rd[j / 2]));
      const int sl = j / (2 * NDB), db = (j / 2) % NDB;
      const unsigned char* base = (second ? Qt : Ot) + ((quarter - 2) * 32 + sl * 16) * ROWB;
      return read_tr_pair(base + tr_lo[db], base + tr_hi[db]);
    };
    auto matrix_step = [&](int k, bf16x8_t op) {
      const int quarter = k / NS, j = k % NS, second = j & 1;
      if (quarter < 2) {
        const int ib = quarter, ks = j / 2;
        floatx16_t zero;
#pragma unroll
        for (int v = 0; v < 16; ++v) zero[v] = 0.f;
        if (second) t[ib] = mfma32(op, vfn[ks], t[ib]);
        else s[ib] = mfma32(op, kf[ks], ks ? s[ib] : zero);
      } else {
        const int ib = quarter - 2, sl = j / (2 * NDB), db = (j / 2) % NDB;
        const uint32_t* w = second ? ew[ib] : pw[ib];
        const bf16x8_t a = as_bf16x8(make_uint4(w[4 * sl], w[4 * sl + 1], w[4 * sl + 2], w[4 * sl + 3]));
        if (second) dk[db] = mfma32(a, op, dk[db]);
        else dv[db] = mfma32(a, op, dv[db]);
      }
    };
    float p_even = 0.f, e_even = 0.f;
    auto element = [&](int ib, int v) {
      const float pv = fast_exp2(fmaf(s[ib][v], p.c, nl[ib][v]));
      const float ev = pv * t[ib][v];
      if (v & 1) {
        pw[ib][v / 2] = pack_bf16x2(p_even, pv);
        ew[ib][v / 2] = pack_bf16x2(e_even, ev);
      } else {
        p_even = pv;
        e_even = ev;
      }
    };
    bf16x8_t ring[2 * PF];
    static_for<0, PF>([&](auto kc) { ring[kc.value] = operand(kc.value); });
    static_for<0, 4 * NS>([&](auto kc) {
      constexpr int k = decltype(kc)::value;
      if constexpr (k % PF == 0) {
        static_for<k + PF, (k + 2 * PF < 4 * NS ? k + 2 * PF : 4 * NS)>(
            [&](auto nc) { ring[nc.value % (2 * PF)] = operand(nc.value); });
      }
      matrix_step(k, ring[k % (2 * PF)]);
      constexpr int quarter = k / NS, j = k % NS;
      if constexpr (quarter == 1 || quarter == 2) {
        static_for<0, EPS>([&](auto uc) { element(quarter - 1, j * EPS + uc.value); });
      }
      __builtin_amdgcn_sched_barrier(0);  // keep the operand reads ahead of their use
    });
    wait_vmcnt<0>();  // this wave's part of the next tile, issued a whole iteration ago
  }

  // ---- dV and dK = -scale * (accumulated E^T Q) of this wave's 32 keys: a lane owns one
  // column per block and 16 key rows
  float* dk_base = p.dk + (((int64_t)b * p.Hkv + hk) * p.kv_len + kseg.start) * D + l32;
  float* dv_base = p.dv + (((int64_t)b * p.Hkv + hk) * p.kv_len + kseg.start) * D + l32;
  const float ns = -p.scale;
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int koff = koff0 + 32 * wave + acc_row(v, hh);
      if (koff < kseg.len) {
        const int64_t o = (int64_t)koff * D + db * 32;
        if (p.add_dkv) {
          unsafeAtomicAdd(dk_base + o, dk[db][v] * ns);
          unsafeAtomicAdd(dv_base + o, dv[db][v]);
        } else {
          dk_base[o] = dk[db][v] * ns;
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
  constexpr int BM = kBwdBM, BN = kBwdBN;
  // Only key tiles that some query can see are listed (eight equal ranges of the list, one
  // per XCD, then carry equal work); key segments nobody sees are cleared by the zero pass.
  // The query-tile loop is spread over several workgroups when the listed tiles are fewer
  // than the CUs, and once more when a diagonal block makes their loop lengths uneven.
  p.kt_total = 0;
  bool diag = false, unseen_keys = false;
  for (int kb = 0; kb < 2; ++kb) {
    bool seen = false;
    if (kb < p.g.nk)
      for (int a = 0; a < p.g.nq; ++a) {
        seen |= p.g.cls[a][kb] != LOONG_SKIP && p.g.q[a].len > 0;
        diag |= p.g.cls[a][kb] == LOONG_DIAG;
      }
    p.nkt[kb] = seen ? (p.g.k[kb].len + BN - 1) / BN : 0;
    p.kt_total += p.nkt[kb];
    unseen_keys |= kb < p.g.nk && !seen && p.g.k[kb].len > 0;
  }
  const int64_t base = (int64_t)p.kt_total * p.Hkv * p.B;
  const int64_t busy = base;
  int nsplit = 1;
  const int64_t q_tiles = std::max<int64_t>((int64_t)p.G * ((p.q_len + BM - 1) / BM), 1);
  if (busy > 0 && busy < 256) nsplit = (int)std::min<int64_t>((256 + busy - 1) / busy, 16);
  if (diag && busy * nsplit <= 512) nsplit *= 2;
  nsplit = (int)std::min<int64_t>(nsplit, q_tiles);
  p.nsplit = nsplit;
  p.add_dkv = (accumulate || nsplit > 1) ? 1 : 0;
  const int64_t total = base * nsplit;
  if (total > 0x3ffffff0) return fail(LOONG_E_UNSUPPORTED, "backward grid too large");
  p.map = make_work_map((int64_t)p.Hkv * p.B, (int64_t)p.kt_total * nsplit);
  if ((nsplit > 1 || unseen_keys) && !accumulate) {
    const int64_t n4 = (int64_t)p.B * p.Hkv * p.kv_len * D / 4;
    zero_kernel<<<dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st>>>(n4, reinterpret_cast<float4*>(p.dk),
                                                                          reinterpret_cast<float4*>(p.dv));
    if (int rc = check_launch("loong_attn_step_bwd (clear dk/dv)")) return rc;
  }
  if (total == 0) return LOONG_OK;
  bwd_dkv_kernel<D><<<dim3(p.map.grid), dim3(kBwdWaves * 64), 0, st>>>(p);
  return check_launch("loong_attn_step_bwd (bf16, dK/dV)");
}

}  // namespace

int launch_bwd_bf16(const loong_step_desc& d, const StepGeom& g, const void* q, const void* k,
                    const void* v, const void* d_o, const float* lse, const float* delta, float* dq,
                    float* dk, float* dv, void* stream) {
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
    const int rc = d.head_dim == 128 ? launch_d<128>(p, accumulate, st) : launch_d<64>(p, accumulate, st);
    if (rc != LOONG_OK) return rc;
  }
  if (d.flags & LOONG_BWD_ONLY_DKV) return LOONG_OK;
  return launch_bwd_dq_bf16(d, g, q, k, v, d_o, lse, delta, dq, stream);
}

}  // namespace loong
