// Centred sliding-window maximum over score rows (the pooling step of the SnapKV
// baseline, Sec. 2.3 / 4.1.1: keep the neighbourhood of strongly attended tokens).
//
// HBM-bound: one read and one write of the [rows, S] fp32 array.  A workgroup
// stages kSegment tokens plus the two halos in LDS (positions outside the row
// hold -inf, which is also what an empty side of the window contributes), then
// every thread takes the maximum over its window from LDS.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "common.h"
#include "kvcrush.h"

namespace {

constexpr int kPoolThreads = 256;
constexpr int kSegment = 2048;     // tokens per workgroup
constexpr int kMaxKernel = 1023;   // halo of at most 511 tokens on each side
constexpr int kStaged = kSegment + kMaxKernel - 1;

__global__ __launch_bounds__(kPoolThreads) void pool_kernel(const float* __restrict__ in,
                                                            float* __restrict__ out, int S, int half,
                                                            int segs_per_row) {
  __shared__ float staged[kStaged];
  const int row = (int)(blockIdx.x / segs_per_row), seg = (int)(blockIdx.x % segs_per_row);
  const int t0 = seg * kSegment;
  const float* src = in + (size_t)row * S;
  const int n_staged = kSegment + 2 * half;
  for (int i = threadIdx.x; i < n_staged; i += kPoolThreads) {
    const int u = t0 - half + i;
    staged[i] = (u >= 0 && u < S) ? src[u] : -INFINITY;
  }
  __syncthreads();
  float* dst = out + (size_t)row * S;
  const int width = 2 * half + 1;
  for (int i = threadIdx.x; i < kSegment; i += kPoolThreads) {
    const int t = t0 + i;
    if (t >= S) break;
    float best = staged[i];
    for (int w = 1; w < width; ++w) best = fmaxf(best, staged[i + w]);
    dst[t] = best;
  }
}

}  // namespace

extern "C" kvcrush_status kvcrush_pool_scores(int32_t rows, int32_t S, int32_t kernel, const float* in,
                                              float* out, void* hip_stream) {
  if (rows < 0 || S < 1 || kernel < 1 || kernel > kMaxKernel || kernel % 2 == 0)
    return KVCRUSH_ERR_INVALID_ARG;
  if (rows == 0) return KVCRUSH_OK;
  if (!in || !out || in == out) return KVCRUSH_ERR_INVALID_ARG;
  const size_t bytes = (size_t)rows * S * sizeof(float);
  const char *a = (const char*)in, *b = (const char*)out;
  if (a < b + bytes && b < a + bytes) return KVCRUSH_ERR_INVALID_ARG;  // overlapping arrays
  const int segs = (S + kSegment - 1) / kSegment;
  if ((long long)rows * segs > 0x7FFFFFFFll) return KVCRUSH_ERR_UNSUPPORTED;
  return kvc::launch(pool_kernel, dim3((unsigned)((long long)rows * segs)), dim3(kPoolThreads), 0,
                     (hipStream_t)hip_stream, in, out, S, kernel / 2, segs);
}
