// Host-only part of the library: error text, descriptor validation, zigzag layout and
// double-ring visit order.  Nothing here touches a device.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "loong_internal.h"

namespace loong {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

void clear_error() { g_err[0] = '\0'; }

static bool mul_ok(int64_t a, int64_t b, int64_t limit) { return a == 0 || b <= limit / a; }

int check_step(const loong_step_desc* d, StepGeom* g) {
  if (!d) return fail(LOONG_E_NULL, "descriptor is NULL");
  if (d->dtype != LOONG_BF16 && d->dtype != LOONG_FP32 && d->dtype != LOONG_FP16)
    return fail(LOONG_E_DTYPE, "dtype %d is none of LOONG_BF16, LOONG_FP32, LOONG_FP16", d->dtype);
  const bool half = d->dtype != LOONG_FP32;  // 16-bit storage: the matrix-core kernels
  if (d->batch < 0 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->head_dim < 1 || d->q_len < 0 ||
      d->kv_len < 0)
    return fail(LOONG_E_SHAPE, "negative size or zero heads (batch %d, heads %d/%d, head_dim %d, q_len %d, kv_len %d)",
                d->batch, d->n_q_heads, d->n_kv_heads, d->head_dim, d->q_len, d->kv_len);
  if (d->n_q_heads % d->n_kv_heads != 0)
    return fail(LOONG_E_UNSUPPORTED, "n_q_heads %d is not a multiple of n_kv_heads %d", d->n_q_heads,
                d->n_kv_heads);
  if (half) {
    if (d->head_dim != 64 && d->head_dim != 128)
      return fail(LOONG_E_UNSUPPORTED, "bf16/fp16 kernels take head_dim 64 or 128, got %d", d->head_dim);
  } else if (d->head_dim > 128 || d->head_dim % 4 != 0) {
    return fail(LOONG_E_UNSUPPORTED, "fp32 kernels take head_dim <= 128 and a multiple of 4, got %d",
                d->head_dim);
  }
  {
    const int forced = (d->flags >> LOONG_KEY_SPLITS_SHIFT) & 7;
    if (forced != 0 && forced != 1 && forced != 2 && forced != 4)
      return fail(LOONG_E_UNSUPPORTED, "LOONG_KEY_SPLITS takes 1, 2 or 4 (0 = automatic), got %d", forced);
  }
  if (!std::isfinite(d->softmax_scale) || d->softmax_scale <= 0.f)
    return fail(LOONG_E_SHAPE, "softmax_scale must be finite and positive");
  const int vec = half ? 8 : 4;  // elements per 16-byte access
  const int64_t* strides[3] = {d->q_stride, d->kv_stride, d->o_stride};
  const int svec[3] = {vec, vec, 4};
  const char* names[3] = {"q_stride", "kv_stride", "o_stride"};
  for (int t = 0; t < 3; ++t)
    for (int i = 0; i < 3; ++i) {
      if (strides[t][i] < 0) return fail(LOONG_E_SHAPE, "%s[%d] is negative", names[t], i);
      if (strides[t][i] % svec[t] != 0)
        return fail(LOONG_E_ALIGN, "%s[%d] = %lld is not a multiple of %d elements", names[t], i,
                    (long long)strides[t][i], svec[t]);
    }
  if (d->q_len > 0 && (d->q_stride[2] < d->head_dim || d->o_stride[2] < d->head_dim))
    return fail(LOONG_E_SHAPE, "token stride of q/out is smaller than head_dim");
  if (d->kv_len > 0 && d->kv_stride[2] < d->head_dim)
    return fail(LOONG_E_SHAPE, "token stride of k/v is smaller than head_dim");
  // the kernels address rows of one tile with 32-bit offsets from a 64-bit tile base
  if (d->q_stride[2] >= (1 << 24) || d->kv_stride[2] >= (1 << 24) || d->o_stride[2] >= (1 << 24))
    return fail(LOONG_E_UNSUPPORTED, "token strides must be below 2^24 elements");
  // keep every row index and every contiguous result offset far inside int64/int32 use
  if (!mul_ok((int64_t)d->batch * d->n_q_heads, (int64_t)d->q_len, (int64_t)1 << 40) ||
      d->q_len > (1 << 24) || d->kv_len > (1 << 24))
    return fail(LOONG_E_UNSUPPORTED, "problem too large (q_len, kv_len <= 2^24; rows <= 2^40)");

  StepGeom geo;
  std::memset(&geo, 0, sizeof(geo));
  if (d->causal) {
    const int c = d->chunk_len;
    if (c < 0 || d->q_len != 2 * c || d->kv_len != 2 * c)
      return fail(LOONG_E_SHAPE, "causal step needs q_len == kv_len == 2*chunk_len (got %d, %d, %d)",
                  d->q_len, d->kv_len, c);
    for (int i = 0; i < 2; ++i)
      if (d->q_chunk[i] < 0 || d->kv_chunk[i] < 0)
        return fail(LOONG_E_SHAPE, "chunk ids must be non-negative");
    if (d->q_chunk[0] == d->q_chunk[1] || d->kv_chunk[0] == d->kv_chunk[1])
      return fail(LOONG_E_SHAPE, "the two halves of a zigzag chunk pair must have different chunk ids");
    geo.nq = geo.nk = 2;
    for (int i = 0; i < 2; ++i) {
      geo.q[i] = Segment{i * c, c, d->q_chunk[i]};
      geo.k[i] = Segment{i * c, c, d->kv_chunk[i]};
    }
    for (int a = 0; a < 2; ++a)
      for (int b = 0; b < 2; ++b)
        geo.cls[a][b] = d->kv_chunk[b] < d->q_chunk[a]    ? LOONG_FULL
                        : d->kv_chunk[b] == d->q_chunk[a] ? LOONG_DIAG
                                                           : LOONG_SKIP;
  } else {
    geo.nq = geo.nk = 1;
    geo.q[0] = Segment{0, d->q_len, 0};
    geo.k[0] = Segment{0, d->kv_len, 0};
    geo.cls[0][0] = LOONG_FULL;
  }
  if (g) *g = geo;
  return LOONG_OK;
}

}  // namespace loong

extern "C" {

const char* loong_last_error(void) { return loong::g_err; }

int loong_version(void) { return 100; }

int loong_validate_step(const loong_step_desc* desc) {
  loong::clear_error();
  return loong::check_step(desc, nullptr);
}

int loong_zigzag_mask(int32_t cp, int32_t inner_w, int32_t rank, int32_t step, int32_t* src_rank,
                      int32_t q_chunk[2], int32_t kv_chunk[2], uint8_t block_class[4]) {
  loong::clear_error();
  if (cp < 1 || inner_w < 1 || cp % inner_w != 0)
    return loong::fail(LOONG_E_SHAPE, "need cp >= 1, inner_w >= 1 and inner_w | cp (cp %d, inner_w %d)", cp,
                       inner_w);
  if (cp > (1 << 29)) return loong::fail(LOONG_E_SHAPE, "cp %d too large", cp);
  if (rank < 0 || rank >= cp || step < 0 || step >= cp)
    return loong::fail(LOONG_E_SHAPE, "rank %d or step %d outside [0, %d)", rank, step, cp);
  // position of this rank on the two rings
  const int32_t rings = cp / inner_w;
  const int32_t ring = rank / inner_w, place = rank % inner_w;
  // micro-step `step` is inner step `hop_in` of outer step `hop_out`; every hop moves a
  // chunk one place forward, so the chunk in hand started that many places behind
  const int32_t hop_out = step / inner_w, hop_in = step % inner_w;
  const int32_t from_ring = (ring - hop_out % rings + rings) % rings;
  const int32_t from_place = (place - hop_in + inner_w) % inner_w;
  const int32_t src = from_ring * inner_w + from_place;
  const int32_t qc[2] = {rank, 2 * cp - 1 - rank};
  const int32_t kc[2] = {src, 2 * cp - 1 - src};
  if (src_rank) *src_rank = src;
  if (q_chunk) { q_chunk[0] = qc[0]; q_chunk[1] = qc[1]; }
  if (kv_chunk) { kv_chunk[0] = kc[0]; kv_chunk[1] = kc[1]; }
  if (block_class)
    for (int a = 0; a < 2; ++a)
      for (int b = 0; b < 2; ++b)
        block_class[a * 2 + b] = kc[b] < qc[a] ? LOONG_FULL : kc[b] == qc[a] ? LOONG_DIAG : LOONG_SKIP;
  return LOONG_OK;
}

}  // extern "C"
