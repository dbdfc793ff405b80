// HBM-bound row kernels of the path: Update (log-sum-exp merge), neutral-element fill,
// output cast and the backward's row term delta = rowsum(dO * O).
#include <hip/hip_runtime.h>

#include "device_utils.h"
#include "loong_internal.h"

namespace loong {

int check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(LOONG_E_HIP, "%s: %s", what, hipGetErrorString(e));
  return LOONG_OK;
}

namespace {

constexpr int kThreads = 256;

// ---- Update(out, lse, block_out, block_lse), Alg. 2 -------------------------------------
// A row is handled by LPR lanes of one wave (LPR a power of two <= 64), each lane moving
// float4 pieces; all lanes of the row read lse before lane 0 of the row rewrites it
// (same wave, program order), so the in-place update has no race.
template <int LPR>
__global__ __launch_bounds__(kThreads) void merge_kernel(int64_t rows, int d4, float* __restrict__ out,
                                                         float* __restrict__ lse,
                                                         const float* __restrict__ bout,
                                                         const float* __restrict__ blse) {
  constexpr int RPB = kThreads / LPR;  // rows per block
  const int sub = threadIdx.x % LPR;
  const int64_t row = (int64_t)blockIdx.x * RPB + threadIdx.x / LPR;
  if (row >= rows) return;
  const float a = lse[row], b = blse[row];
  const float hi = fmaxf(a, b);
  if (b == -INFINITY) return;  // nothing arrives: running result stays as it is
  // weights of the two sides; hi is finite here because b is
  const float ea = fast_exp2((a - hi) * kLog2e), eb = fast_exp2((b - hi) * kLog2e);
  const float tot = ea + eb;
  const float wa = ea / tot, wb = eb / tot;
  const bool fresh = a == -INFINITY;  // running side empty: take the arriving rows as they are
  float4* o4 = reinterpret_cast<float4*>(out) + row * d4;
  const float4* b4 = reinterpret_cast<const float4*>(bout) + row * d4;
  for (int c = sub; c < d4; c += LPR) {
    float4 x = o4[c];
    const float4 y = b4[c];
    x.x = fresh ? y.x : wa * x.x + wb * y.x;
    x.y = fresh ? y.y : wa * x.y + wb * y.y;
    x.z = fresh ? y.z : wa * x.z + wb * y.z;
    x.w = fresh ? y.w : wa * x.w + wb * y.w;
    o4[c] = x;
  }
  if (sub == 0) lse[row] = hi + fast_log2(tot) * kLn2;
}

__global__ __launch_bounds__(kThreads) void init_running_kernel(int64_t n4, int64_t rows, float4* out,
                                                                float* lse) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < n4) out[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  if (i < rows) lse[i] = -INFINITY;
}

// fp32 -> bf16 or fp16, eight elements per thread; or plain copy for fp32 storage (four per thread)
template <class E>
__global__ __launch_bounds__(kThreads) void cast_half_kernel(int64_t n8, const float4* __restrict__ in,
                                                             uint4* __restrict__ o) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= n8) return;
  const float4 a = in[2 * i], b = in[2 * i + 1];
  o[i] = make_uint4(E::pack2(a.x, a.y), E::pack2(a.z, a.w), E::pack2(b.x, b.y), E::pack2(b.z, b.w));
}

__global__ __launch_bounds__(kThreads) void copy_f32_kernel(int64_t n4, const float4* __restrict__ in,
                                                            float4* __restrict__ o) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < n4) o[i] = in[i];
}

// ---- delta_i = sum_k dO_ik O_ik ----------------------------------------------------------
// LPR lanes per row, each lane 16 bytes at a time; rows are (batch, head, token) with strides.
template <class E, int LPR>  // E = Bf16, Fp16, or float for fp32 storage
__global__ __launch_bounds__(kThreads) void delta_kernel(int64_t rows, int heads, int len, int dvec,
                                                         int64_t s0, int64_t s1, int64_t s2,
                                                         const void* __restrict__ o_,
                                                         const void* __restrict__ do_,
                                                         float* __restrict__ delta) {
  constexpr int RPB = kThreads / LPR;
  const int sub = threadIdx.x % LPR;
  int64_t row = (int64_t)blockIdx.x * RPB + threadIdx.x / LPR;
  const bool live = row < rows;
  if (!live) row = rows - 1;  // keep the whole wave in the shuffle below
  const int t = (int)(row % len);
  const int h = (int)((row / len) % heads);
  const int64_t b = row / ((int64_t)len * heads);
  const int64_t base = b * s0 + h * s1 + t * s2;
  float acc = 0.f;
  for (int c = sub; c < dvec; c += LPR) {
    if constexpr (!std::is_same<E, float>::value) {
      const uint4 x = reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(o_) + base)[c];
      const uint4 y = reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(do_) + base)[c];
      acc += E::lo(x.x) * E::lo(y.x) + E::hi(x.x) * E::hi(y.x);
      acc += E::lo(x.y) * E::lo(y.y) + E::hi(x.y) * E::hi(y.y);
      acc += E::lo(x.z) * E::lo(y.z) + E::hi(x.z) * E::hi(y.z);
      acc += E::lo(x.w) * E::lo(y.w) + E::hi(x.w) * E::hi(y.w);
    } else {
      const float4 x = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(o_) + base)[c];
      const float4 y = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(do_) + base)[c];
      acc += x.x * y.x + x.y * y.y + x.z * y.z + x.w * y.w;
    }
  }
#pragma unroll
  for (int m = LPR / 2; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
  if (live && sub == 0) delta[row] = acc;
}

int pow2_lanes(int pieces) {
  int l = 1;
  while (l < pieces && l < 64) l <<= 1;
  return l;
}

int64_t blocks_for(int64_t items, int per_block) { return (items + per_block - 1) / per_block; }

}  // namespace
}  // namespace loong

using namespace loong;

extern "C" {

int loong_lse_merge(int64_t rows, int32_t head_dim, float* out, float* lse, const float* block_out,
                    const float* block_lse, void* stream) {
  clear_error();
  if (!out || !lse || !block_out || !block_lse) return fail(LOONG_E_NULL, "loong_lse_merge: NULL tensor");
  if (rows < 0 || head_dim < 1) return fail(LOONG_E_SHAPE, "loong_lse_merge: rows %lld, head_dim %d", (long long)rows, head_dim);
  if (head_dim % 4 != 0) return fail(LOONG_E_UNSUPPORTED, "loong_lse_merge: head_dim %d is not a multiple of 4", head_dim);
  if (!aligned16(out) || !aligned16(block_out)) return fail(LOONG_E_ALIGN, "loong_lse_merge: out/block_out not 16-byte aligned");
  if (rows > ((int64_t)1 << 40)) return fail(LOONG_E_UNSUPPORTED, "loong_lse_merge: too many rows");
  if (rows == 0) return LOONG_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int d4 = head_dim / 4;
  const int lpr = pow2_lanes(d4);
  const int64_t nb = blocks_for(rows, kThreads / lpr);
  if (nb > 0x7fffffff) return fail(LOONG_E_UNSUPPORTED, "loong_lse_merge: grid too large");
  dim3 grid((unsigned)nb), block(kThreads);
  switch (lpr) {
    case 1: merge_kernel<1><<<grid, block, 0, st>>>(rows, d4, out, lse, block_out, block_lse); break;
    case 2: merge_kernel<2><<<grid, block, 0, st>>>(rows, d4, out, lse, block_out, block_lse); break;
    case 4: merge_kernel<4><<<grid, block, 0, st>>>(rows, d4, out, lse, block_out, block_lse); break;
    case 8: merge_kernel<8><<<grid, block, 0, st>>>(rows, d4, out, lse, block_out, block_lse); break;
    case 16: merge_kernel<16><<<grid, block, 0, st>>>(rows, d4, out, lse, block_out, block_lse); break;
    case 32: merge_kernel<32><<<grid, block, 0, st>>>(rows, d4, out, lse, block_out, block_lse); break;
    default: merge_kernel<64><<<grid, block, 0, st>>>(rows, d4, out, lse, block_out, block_lse); break;
  }
  return check_launch("loong_lse_merge");
}

int loong_init_running(int64_t rows, int32_t head_dim, float* out, float* lse, void* stream) {
  clear_error();
  if (!out || !lse) return fail(LOONG_E_NULL, "loong_init_running: NULL tensor");
  if (rows < 0 || head_dim < 1) return fail(LOONG_E_SHAPE, "loong_init_running: rows %lld, head_dim %d", (long long)rows, head_dim);
  if (head_dim % 4 != 0) return fail(LOONG_E_UNSUPPORTED, "loong_init_running: head_dim %d is not a multiple of 4", head_dim);
  if (!aligned16(out)) return fail(LOONG_E_ALIGN, "loong_init_running: out not 16-byte aligned");
  if (rows > ((int64_t)1 << 40)) return fail(LOONG_E_UNSUPPORTED, "loong_init_running: too many rows");
  if (rows == 0) return LOONG_OK;
  const int64_t n4 = rows * (head_dim / 4);
  const int64_t nb = blocks_for(n4, kThreads);
  if (nb > 0x7fffffff) return fail(LOONG_E_UNSUPPORTED, "loong_init_running: grid too large");
  init_running_kernel<<<dim3((unsigned)nb), dim3(kThreads), 0, static_cast<hipStream_t>(stream)>>>(
      n4, rows, reinterpret_cast<float4*>(out), lse);
  return check_launch("loong_init_running");
}

int loong_finalize_out(int64_t rows, int32_t head_dim, const float* out, void* o, int32_t dtype,
                       void* stream) {
  clear_error();
  if (!out || !o) return fail(LOONG_E_NULL, "loong_finalize_out: NULL tensor");
  if (dtype != LOONG_BF16 && dtype != LOONG_FP32 && dtype != LOONG_FP16)
    return fail(LOONG_E_DTYPE, "loong_finalize_out: dtype %d", dtype);
  if (rows < 0 || head_dim < 1) return fail(LOONG_E_SHAPE, "loong_finalize_out: rows %lld, head_dim %d", (long long)rows, head_dim);
  const int vec = dtype == LOONG_FP32 ? 4 : 8;
  if (head_dim % vec != 0) return fail(LOONG_E_UNSUPPORTED, "loong_finalize_out: head_dim %d is not a multiple of %d", head_dim, vec);
  if (!aligned16(out) || !aligned16(o)) return fail(LOONG_E_ALIGN, "loong_finalize_out: pointers not 16-byte aligned");
  if (rows > ((int64_t)1 << 40)) return fail(LOONG_E_UNSUPPORTED, "loong_finalize_out: too many rows");
  if (rows == 0) return LOONG_OK;
  const int64_t n = rows * (head_dim / vec);
  const int64_t nb = blocks_for(n, kThreads);
  if (nb > 0x7fffffff) return fail(LOONG_E_UNSUPPORTED, "loong_finalize_out: grid too large");
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (dtype == LOONG_BF16)
    cast_half_kernel<Bf16><<<dim3((unsigned)nb), dim3(kThreads), 0, st>>>(n, reinterpret_cast<const float4*>(out),
                                                                         reinterpret_cast<uint4*>(o));
  else if (dtype == LOONG_FP16)
    cast_half_kernel<Fp16><<<dim3((unsigned)nb), dim3(kThreads), 0, st>>>(n, reinterpret_cast<const float4*>(out),
                                                                         reinterpret_cast<uint4*>(o));
  else
    copy_f32_kernel<<<dim3((unsigned)nb), dim3(kThreads), 0, st>>>(n, reinterpret_cast<const float4*>(out),
                                                                  reinterpret_cast<float4*>(o));
  return check_launch("loong_finalize_out");
}

int loong_bwd_delta(const loong_step_desc* desc, const void* o, const void* d_o, float* delta,
                    void* stream) {
  clear_error();
  if (int rc = check_step(desc, nullptr)) return rc;
  if (!o || !d_o || !delta) return fail(LOONG_E_NULL, "loong_bwd_delta: NULL tensor");
  if (!aligned16(o) || !aligned16(d_o)) return fail(LOONG_E_ALIGN, "loong_bwd_delta: o/d_o not 16-byte aligned");
  const int64_t rows = (int64_t)desc->batch * desc->n_q_heads * desc->q_len;
  if (rows == 0) return LOONG_OK;
  const int dvec = desc->head_dim / (desc->dtype == LOONG_FP32 ? 4 : 8);
  const int lpr = pow2_lanes(dvec);
  const int64_t nb = blocks_for(rows, kThreads / lpr);
  if (nb > 0x7fffffff) return fail(LOONG_E_UNSUPPORTED, "loong_bwd_delta: grid too large");
  dim3 grid((unsigned)nb), block(kThreads);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int64_t* s = desc->q_stride;
#define LOONG_DELTA(BF, L)                                                                               \
  delta_kernel<BF, L><<<grid, block, 0, st>>>(rows, desc->n_q_heads, desc->q_len, dvec, s[0], s[1], s[2], \
                                               o, d_o, delta)
#define LOONG_DELTA_L(BF)              \
  switch (lpr) {                       \
    case 1: LOONG_DELTA(BF, 1); break; \
    case 2: LOONG_DELTA(BF, 2); break; \
    case 4: LOONG_DELTA(BF, 4); break; \
    case 8: LOONG_DELTA(BF, 8); break; \
    case 16: LOONG_DELTA(BF, 16); break; \
    default: LOONG_DELTA(BF, 32); break; \
  }
  if (desc->dtype == LOONG_BF16) { LOONG_DELTA_L(Bf16) } else if (desc->dtype == LOONG_FP16) { LOONG_DELTA_L(Fp16) } else { LOONG_DELTA_L(float) }
#undef LOONG_DELTA_L
#undef LOONG_DELTA
  return check_launch("loong_bwd_delta");
}

}  // extern "C"

// ---- measurement aid: matrix cores only ---------------------------------------------------
namespace loong {
namespace {
__global__ __launch_bounds__(256) void mfma_probe_kernel(int iters, const uint4* operands, float* sink) {
  const int lane = threadIdx.x & 63;
  // built-in operands: nearly constant (few bits change from lane to lane), accumulators stay finite
  bf16x8_t a = as_bf16x8(make_uint4(0x3c003c00u + lane, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u));
  bf16x8_t b = as_bf16x8(make_uint4(0x38003800u, 0x38003800u + lane, 0x38003800u, 0x38003800u));
  if (operands) {  // the caller's values: what the clocks do depends on how many bits toggle
    a = as_bf16x8(operands[lane]);
    b = as_bf16x8(operands[64 + lane]);
  }
  floatx16_t c[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) c[i][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i) c[i] = mfma32(a, b, c[i]);
  }
  sink[blockIdx.x * 256 + threadIdx.x] = c[0][0] + c[1][5] + c[2][10] + c[3][15];
}
}  // namespace
}  // namespace loong

extern "C" int loong_mfma_probe(int32_t workgroups, int32_t iters, const void* operands, float* sink, void* stream) {
  loong::clear_error();
  if (!sink) return loong::fail(LOONG_E_NULL, "loong_mfma_probe: NULL sink");
  if (workgroups <= 0 || iters <= 0) return loong::fail(LOONG_E_SHAPE, "loong_mfma_probe: sizes must be positive");
  if (operands && (reinterpret_cast<uintptr_t>(operands) & 15)) return loong::fail(LOONG_E_ALIGN, "loong_mfma_probe: operands must be 16-byte aligned");
  loong::mfma_probe_kernel<<<dim3((unsigned)workgroups), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(
      iters, static_cast<const uint4*>(operands), sink);
  return loong::check_launch("loong_mfma_probe");
}
