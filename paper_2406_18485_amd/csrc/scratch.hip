// loong_attn_step_bwd_static: the backward micro-step for callers that cannot allocate device
// memory (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
// The scratch of the dK/dV kernel (arrival counters and the partial sums of shared query loops)
// lives in a device array that is part of the library's code object instead of a buffer the
// caller brings: every GPU the library runs on holds its own copy from the first use of the
// library on it until the process ends.
#include <hip/hip_runtime.h>

#include <atomic>

#include "loong_internal.h"

namespace {

// counters + 64 MiB of partial sums: enough for every step of the 32K..1M-token benchmark shapes
// (at most 512 (key tile, split) slots of 128 KiB)
constexpr int64_t kScratchBytes = LOONG_STATIC_SCRATCH_BYTES;
static_assert(kScratchBytes == loong::kWsHeadBytes + ((int64_t)64 << 20), "header and layout disagree");

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
// device address of `scratch` on each device, looked up once per device with that device current
std::atomic<void*> g_scratch_ptr[kMaxDevices];

int scratch_address(void** ptr) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return loong::fail(LOONG_E_HIP, "loong_attn_step_bwd_static: no current HIP device");
  }
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      (void)hipGetLastError();
      return loong::fail(LOONG_E_HIP, "loong_attn_step_bwd_static: cannot locate the scratch array on device %d: %s", dev,
                         hipGetErrorString(e));
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  return LOONG_OK;
}

}  // namespace

extern "C" {

__attribute__((visibility("default"))) int loong_attn_step_bwd_static(const loong_step_desc* desc, const void* q, const void* k,
                                                                      const void* v, const void* o, const void* d_o,
                                                                      const float* lse, float* delta, float* dq, float* dk,
                                                                      float* dv, void* stream) {
  loong::clear_error();
  int64_t need = 0;
  if (int rc = loong_workspace_bytes(desc, &need)) return rc;
  if (need > kScratchBytes)
    return loong::fail(LOONG_E_UNSUPPORTED,
                       "loong_attn_step_bwd_static: this step needs %lld bytes of scratch, the static array holds %lld; "
                       "use loong_attn_step_bwd with a workspace of the caller's",
                       (long long)need, (long long)kScratchBytes);
  void* ptr = nullptr;
  if (need > 0)
    if (int rc = scratch_address(&ptr)) return rc;
  return loong_attn_step_bwd(desc, q, k, v, o, d_o, lse, delta, dq, dk, dv, ptr, need > 0 ? kScratchBytes : 0, stream);
}

}  // extern "C"
