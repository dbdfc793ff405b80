// Layout steps either side of the ring (Alg. 1): the local re-arrangements of SeqAlltoAll and
// the KV replication of GQA as one strided row copy, and the reduction of the replicated heads'
// gradients.  HBM-bound: every byte is read once and written once, 16 bytes per lane.
#include <hip/hip_runtime.h>

#include "loong_internal.h"

namespace loong {
namespace {

struct PermuteParams {
  int64_t n1, n2, pieces;            // rows are indexed (a, b, c), each `pieces` 16-byte pieces long
  int64_t is0, is1, is2, os0, os1, os2;
  int64_t total;                     // pieces to copy
};

__global__ __launch_bounds__(256) void permute_rows_kernel(PermuteParams p, const unsigned char* in, unsigned char* out) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= p.total) return;
  const int64_t row = i / p.pieces, piece = i - row * p.pieces;
  const int64_t ab = row / p.n2, c = row - ab * p.n2;
  const int64_t a = ab / p.n1, b = ab - a * p.n1;
  const uint4 v = *reinterpret_cast<const uint4*>(in + a * p.is0 + b * p.is1 + c * p.is2 + piece * 16);
  *reinterpret_cast<uint4*>(out + a * p.os0 + b * p.os1 + c * p.os2 + piece * 16) = v;
}

__global__ __launch_bounds__(256) void reduce_replicas_kernel(int64_t heads, int rep, int64_t quads_per_head,
                                                              const float4* in, float4* out) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= heads * quads_per_head) return;
  const int64_t h = i / quads_per_head, q = i - h * quads_per_head;
  const float4* src = in + (h * rep) * quads_per_head + q;
  float4 acc = src[0];
  for (int r = 1; r < rep; ++r) {
    const float4 x = src[(int64_t)r * quads_per_head];
    acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
  }
  out[i] = acc;
}

}  // namespace
}  // namespace loong

using namespace loong;

extern "C" {

int loong_permute_rows(const int64_t n[3], const int64_t in_stride[3], const int64_t out_stride[3], int64_t row_bytes,
                       const void* in, void* out, void* stream) {
  clear_error();
  if (!n || !in_stride || !out_stride || !in || !out) return fail(LOONG_E_NULL, "loong_permute_rows: NULL argument");
  if (n[0] < 0 || n[1] < 0 || n[2] < 0 || row_bytes < 0) return fail(LOONG_E_SHAPE, "loong_permute_rows: negative size");
  if (row_bytes % 16 != 0 || !aligned16(in) || !aligned16(out))
    return fail(LOONG_E_ALIGN, "loong_permute_rows: rows must be 16-byte aligned multiples of 16 bytes");
  for (int i = 0; i < 3; ++i) {
    if (in_stride[i] < 0 || out_stride[i] < 0) return fail(LOONG_E_SHAPE, "loong_permute_rows: negative stride");
    if (in_stride[i] % 16 != 0 || out_stride[i] % 16 != 0)
      return fail(LOONG_E_ALIGN, "loong_permute_rows: strides must be multiples of 16 bytes");
  }
  PermuteParams p{};
  p.n1 = n[1]; p.n2 = n[2]; p.pieces = row_bytes / 16;
  p.is0 = in_stride[0]; p.is1 = in_stride[1]; p.is2 = in_stride[2];
  p.os0 = out_stride[0]; p.os1 = out_stride[1]; p.os2 = out_stride[2];
  p.total = n[0] * n[1] * n[2] * p.pieces;
  if (p.total == 0) return LOONG_OK;
  const int64_t blocks = (p.total + 255) / 256;
  if (blocks > 0x7fffffff) return fail(LOONG_E_UNSUPPORTED, "loong_permute_rows: more than 2^31-1 workgroups");
  permute_rows_kernel<<<dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(
      p, static_cast<const unsigned char*>(in), static_cast<unsigned char*>(out));
  return check_launch("loong_permute_rows");
}

int loong_reduce_replicas(int64_t heads, int32_t rep, int64_t elems_per_head, const float* in, float* out, void* stream) {
  clear_error();
  if (!in || !out) return fail(LOONG_E_NULL, "loong_reduce_replicas: NULL tensor");
  if (heads < 0 || rep < 1 || elems_per_head < 0) return fail(LOONG_E_SHAPE, "loong_reduce_replicas: bad sizes");
  if (elems_per_head % 4 != 0 || !aligned16(in) || !aligned16(out))
    return fail(LOONG_E_ALIGN, "loong_reduce_replicas: elems_per_head must be a multiple of 4, pointers 16-byte aligned");
  const int64_t total = heads * (elems_per_head / 4);
  if (total == 0) return LOONG_OK;
  const int64_t blocks = (total + 255) / 256;
  if (blocks > 0x7fffffff) return fail(LOONG_E_UNSUPPORTED, "loong_reduce_replicas: more than 2^31-1 workgroups");
  reduce_replicas_kernel<<<dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(
      heads, rep, elems_per_head / 4, reinterpret_cast<const float4*>(in), reinterpret_cast<float4*>(out));
  return check_launch("loong_reduce_replicas");
}

}  // extern "C"
