// Internal helpers shared by the gfx950 kernels of libkvcrush (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvcrush.h"

#define KVC_WAVE 64

namespace kvc {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Launch-status check that does not synchronise.
inline kvcrush_status launch_status() {
  return hipGetLastError() == hipSuccess ? KVCRUSH_OK : KVCRUSH_ERR_HIP;
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (KVC_WAVE - 1)); }

__device__ __forceinline__ uint64_t lanemask_lt() {
  return (1ull << lane_id()) - 1ull;
}

}  // namespace kvc
