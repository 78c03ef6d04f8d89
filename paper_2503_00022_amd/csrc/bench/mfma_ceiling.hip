// Measurement aid, not part of libkvcrush: what the matrix pipe of this chip sustains on
// v_mfma_f32_32x32x16_bf16 alone, with operands of the benchmark's own value distribution
// (operand toggling moves the power-limited clock), no LDS traffic and no vector ALU work.
// bench.py reports it beside the datasheet peak as the ceiling stage 1 could reach if its
// exponentials and tile traffic were free.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;   // four waves a workgroup, two workgroups a compute unit, as the score kernels
constexpr int kFrags = 8;       // operand fragments a wave cycles through (one head row block at D = 128)
constexpr int kMfmaPerIter = 2 * kFrags;

// operands: at least kThreads * kFrags * 2 * 16 bytes of bf16 values.  out: gridDim.x * kThreads floats.
__global__ __launch_bounds__(kThreads, 2) void mfma_ceiling_kernel(const u32x4* __restrict__ operands, int iters,
                                                                   float* __restrict__ out) {
  u32x4 a[kFrags], b[kFrags];
#pragma unroll
  for (int s = 0; s < kFrags; ++s) {
    a[s] = operands[(2 * s) * kThreads + threadIdx.x];
    b[s] = operands[(2 * s + 1) * kThreads + threadIdx.x];
  }
  f32x16 acc0 = {0}, acc1 = {0};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int s = 0; s < kFrags; ++s) {
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[s]), __builtin_bit_cast(bf16x8, b[s]),
                                                     acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[(s + 3) % kFrags]),
                                                     __builtin_bit_cast(bf16x8, b[s]), acc1, 0, 0, 0);
    }
  }
  float v = 0.0f;
#pragma unroll
  for (int r = 0; r < 16; ++r) v += acc0[r] + acc1[r];
  out[(size_t)blockIdx.x * kThreads + threadIdx.x] = v;
}

}  // namespace

// Enqueues one launch on `hip_stream`.  operands: device, >= kvcrush_bench_mfma_operand_bytes() bytes of
// bf16 values; out: device, grid * 256 floats.  Returns the floating-point operations of the launch
// (0 on a bad argument or a refused launch).
extern "C" double kvcrush_bench_mfma_ceiling(const void* operands, int32_t iters, int32_t grid, float* out,
                                             void* hip_stream) {
  if (!operands || !out || iters < 1 || grid < 1) return 0.0;
  hipLaunchKernelGGL(mfma_ceiling_kernel, dim3((unsigned)grid), dim3(kThreads), 0, (hipStream_t)hip_stream,
                     (const u32x4*)operands, iters, out);
  if (hipGetLastError() != hipSuccess) return 0.0;
  return (double)grid * (kThreads / 64) * (double)iters * kMfmaPerIter * (2.0 * 32 * 32 * 16);
}

extern "C" size_t kvcrush_bench_mfma_operand_bytes(void) { return (size_t)kThreads * kFrags * 2 * sizeof(u32x4); }
