// Device memory the library owns for partial results that workgroups of one launch hand to
// each other: one block per device, grown on demand, kept until the process ends.  Layout:
// kWsCounters zero-initialised 32-bit counters (every user leaves them at zero), then the
// payload.  All launches that use it on one device must be ordered on one stream: they share
// the block.
#include <hip/hip_runtime.h>

#include <mutex>

#include "loong_internal.h"

namespace loong {
namespace {

struct Block {
  void* base = nullptr;
  size_t payload = 0;
};

constexpr int kMaxDevices = 64;
Block g_blocks[kMaxDevices];
std::mutex g_mutex;

}  // namespace

int workspace_get(size_t payload_bytes, uint32_t** counters, float** payload) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    return fail(LOONG_E_HIP, "workspace: no current device");
  std::lock_guard<std::mutex> lock(g_mutex);
  Block& blk = g_blocks[dev];
  if (!blk.base || blk.payload < payload_bytes) {
    // growing: nothing of ours may still be using the old block
    if (blk.base) {
      if (hipDeviceSynchronize() != hipSuccess || hipFree(blk.base) != hipSuccess)
        return fail(LOONG_E_HIP, "workspace: cannot release the old block: %s", hipGetErrorString(hipGetLastError()));
      blk = Block{};
    }
    const size_t head = (size_t)kWsCounters * sizeof(uint32_t);
    void* mem = nullptr;
    hipError_t e = hipMalloc(&mem, head + payload_bytes);
    if (e == hipSuccess) e = hipMemset(mem, 0, head);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
      (void)hipGetLastError();
      if (mem) (void)hipFree(mem);
      return fail(LOONG_E_HIP,
                  "workspace: cannot allocate %zu bytes (%s); under stream capture reserve it beforehand with "
                  "loong_reserve_workspace",
                  head + payload_bytes, hipGetErrorString(e));
    }
    blk.base = mem;
    blk.payload = payload_bytes;
  }
  *counters = static_cast<uint32_t*>(blk.base);
  *payload = reinterpret_cast<float*>(static_cast<unsigned char*>(blk.base) + (size_t)kWsCounters * sizeof(uint32_t));
  return LOONG_OK;
}

}  // namespace loong

extern "C" __attribute__((visibility("default"))) int loong_reserve_workspace(int64_t bytes) {
  loong::clear_error();
  if (bytes < 0 || bytes > ((int64_t)1 << 34)) return loong::fail(LOONG_E_SHAPE, "loong_reserve_workspace: %lld bytes", (long long)bytes);
  uint32_t* c;
  float* p;
  return loong::workspace_get((size_t)bytes, &c, &p);
}
