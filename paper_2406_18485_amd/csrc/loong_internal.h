// Internal declarations shared by the host side of the library (not part of the ABI).
#pragma once
#include <stddef.h>
#include <stdint.h>
#include "loong.h"

namespace loong {

// Record an error text for the calling thread and hand back `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

// A run of consecutive local tokens that belong to one global chunk.
struct Segment {
  int32_t start;   // first local token
  int32_t len;     // tokens
  int32_t chunk;   // global chunk id (only compared, never used as an address)
};

// Geometry of one micro-step after validation: up to two q segments and two key
// segments, and the class of every (q segment, key segment) block.
struct StepGeom {
  int32_t nq, nk;
  Segment q[2], k[2];
  uint8_t cls[2][2];
};

// Validate a descriptor (no device access).  Fills `g` when it succeeds.
int check_step(const loong_step_desc* d, StepGeom* g);

// 16-byte alignment test for device pointers.
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Map a hipError_t (as int) of the last launch to the ABI status.
int check_launch(const char* what);

// Facts of the current device, looked up once per device (device.hip).  device_facts fails with
// LOONG_E_HIP when there is no device and LOONG_E_UNSUPPORTED when it is not a gfx950 part.
struct DeviceFacts {
  int cus;  // compute units
};
int device_facts(DeviceFacts* f);
// Compute units to plan a launch for: the current device's, or those of an MI355X when no
// device can be asked (host-only size queries on a machine without a GPU).
constexpr int kDefaultCus = 256;
int planning_cus();

// Workspace of the backward step (caller-owned device memory): kWsCounters 32-bit arrival
// counters, then the partial sums.  The step clears the counters it uses with a kernel of its
// own before the kernel that counts, so the memory may hold anything when it is handed in.
constexpr int kWsCounters = 16384;
constexpr int64_t kWsHeadBytes = (int64_t)kWsCounters * 4;

// Key splits of the row-owning kernels forced through the descriptor's flags (0: automatic).
inline int forced_key_splits(int flags) {
  const int v = (flags >> LOONG_KEY_SPLITS_SHIFT) & 7;
  return v == 1 || v == 2 || v == 4 ? v : 0;
}

}  // namespace loong

// Kernel launchers (defined next to their kernels).  All arguments are already validated.
// The *_bf16 launchers serve both 16-bit storage types (LOONG_BF16 and LOONG_FP16).
namespace loong {
int launch_fwd_f32(const loong_step_desc& d, const StepGeom& g, const void* q, const void* k,
                   const void* v, float* out, float* lse, void* stream);
int launch_bwd_f32(const loong_step_desc& d, const StepGeom& g, const void* q, const void* k,
                   const void* v, const void* d_o, const float* lse, const float* delta, float* dq,
                   float* dk, float* dv, void* stream);
int launch_fwd_bf16(const loong_step_desc& d, const StepGeom& g, const void* q, const void* k,
                    const void* v, float* out, float* lse, void* stream);
int launch_bwd_bf16(const loong_step_desc& d, const StepGeom& g, const void* q, const void* k,
                    const void* v, const void* d_o, const float* lse, const float* delta, float* dq,
                    float* dk, float* dv, void* workspace, int64_t workspace_bytes, void* stream);
int64_t bwd_workspace_bytes_bf16(const loong_step_desc& d, const StepGeom& g);
int launch_bwd_dq_bf16(const loong_step_desc& d, const StepGeom& g, const void* q, const void* k,
                       const void* v, const void* d_o, const float* lse, const float* delta, float* dq,
                       void* stream);
}  // namespace loong
