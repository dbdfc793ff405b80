// What the launch planning needs to know about the current device: that it is a gfx950 part
// (the kernels are written for its matrix instructions, LDS size and eight XCDs) and how many
// compute units it has.  The facts of a device never change, so each is looked up once and
// remembered (a write-once table; no other state is kept in the library).
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstring>

#include "loong_internal.h"

namespace loong {
namespace {

constexpr int kMaxDevices = 64;
// 0: not looked up yet; > 0: compute units of a gfx950 device; -1: another architecture
std::atomic<int> g_cus[kMaxDevices];

}  // namespace

int device_facts(DeviceFacts* f) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return fail(LOONG_E_HIP, "no current HIP device");
  }
  int cus = g_cus[dev].load(std::memory_order_acquire);
  if (cus == 0) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) {
      (void)hipGetLastError();
      return fail(LOONG_E_HIP, "cannot read the properties of device %d", dev);
    }
    cus = std::strncmp(prop.gcnArchName, "gfx950", 6) == 0 && prop.multiProcessorCount > 0 ? prop.multiProcessorCount : -1;
    g_cus[dev].store(cus, std::memory_order_release);
  }
  if (cus < 0) return fail(LOONG_E_UNSUPPORTED, "device %d is not a gfx950 part: the kernels are built for gfx950 only", dev);
  f->cus = cus;
  return LOONG_OK;
}

int planning_cus() {
  DeviceFacts f;
  if (device_facts(&f) == LOONG_OK) return f.cus;
  clear_error();
  return kDefaultCus;
}

}  // namespace loong
