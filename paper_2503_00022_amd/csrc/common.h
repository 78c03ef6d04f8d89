// Internal helpers shared by the gfx950 kernels of libkvcrush (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <tuple>
#include <utility>

#include "kvcrush.h"

#define KVC_WAVE 64

namespace kvc {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Kernel launch whose status is this launch's own: an error left behind by an earlier,
// unrelated runtime call is neither reported nor cleared.  Does not synchronise.
template <typename... KArgs, size_t... I>
inline hipError_t launch_impl(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t dynamic_lds,
                              hipStream_t stream, std::tuple<KArgs...>& vals, std::index_sequence<I...>) {
  void* args[] = {static_cast<void*>(&std::get<I>(vals))...};
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, args, dynamic_lds, stream);
}
template <typename... KArgs, typename... Args>
inline kvcrush_status launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t dynamic_lds,
                             hipStream_t stream, const Args&... args) {
  static_assert(sizeof...(KArgs) == sizeof...(Args), "one value per kernel parameter");
  std::tuple<KArgs...> vals(args...);
  return launch_impl(kernel, grid, block, dynamic_lds, stream, vals, std::index_sequence_for<KArgs...>{}) == hipSuccess
             ? KVCRUSH_OK
             : KVCRUSH_ERR_HIP;
}

// Dynamic LDS beyond the default limit has to be allowed per kernel; done once per kernel
// and device (to the most a workgroup can have beside `static_lds` bytes of static arrays),
// not on every call.
constexpr int kLdsPerWorkgroup = 160 * 1024;
template <auto Kernel>
inline kvcrush_status allow_large_lds(int static_lds) {
  static std::atomic<uint64_t> done{0};  // one bit per device
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return KVCRUSH_ERR_HIP;
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return KVCRUSH_OK;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          kLdsPerWorkgroup - static_lds) != hipSuccess)
    return KVCRUSH_ERR_HIP;
  done.fetch_or(bit, std::memory_order_release);
  return KVCRUSH_OK;
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (KVC_WAVE - 1)); }

__device__ __forceinline__ uint64_t lanemask_lt() {
  return (1ull << lane_id()) - 1ull;
}

}  // namespace kvc
