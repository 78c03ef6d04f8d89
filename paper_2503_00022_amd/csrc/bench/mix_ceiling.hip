// Measurement aid, not part of libkvcrush: what this chip sustains on the score kernels'
// own instruction mix with everything else taken away.  Per step a wave issues 16
// v_mfma_f32_32x32x16_bf16 (one 64 x 32 block of Q K^T at D = 128) and, for each of the 32
// accumulator values of the PREVIOUS block, the three vector-ALU instructions every score
// element costs (multiply-add by the softmax scale, exp2, add into a running sum), in the
// same interleave as the kernels' hand-written pipeline (every MFMA followed by its share of the
// vector work).  No global or LDS traffic inside the loop, two waves per SIMD like the score
// kernels, operands taken from the benchmark's own Q values.  Matrix-core and vector
// instructions of a SIMD share one issue port, so this mix runs below the MFMA-only ceiling
// (csrc/bench/mfma_ceiling.hip); bench.py reports both beside the datasheet peak.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;  // four waves a workgroup, two workgroups a compute unit
constexpr int kSteps = 8;      // MFMA steps per 32 x 32 tile at D = 128
constexpr int kSchedMfma = 0x008, kSchedValu = 0x002 | 0x400;

// One block: the MFMAs of acc_new, and exp2(acc_old * c - ref) added into col.
__device__ __forceinline__ void mix_half(f32x16 (&acc_new)[2], const f32x16 (&acc_old)[2], f32x16 (&col)[2],
                                         const u32x4 (&a0)[kSteps], const u32x4 (&a1)[kSteps],
                                         u32x4 (&b)[kSteps], float c, float ref) {
  constexpr int kPer = 32 / kSteps;  // elements of acc_old per MFMA pair
  // The operands never change, so without this the compiler would compute the block once and
  // reuse it: an empty statement that claims to rewrite two operand registers keeps every
  // block's MFMAs in the loop, at no instruction's cost.
  asm volatile("" : "+v"(b[0]), "+v"(b[kSteps - 1]));
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_new[t][r] = 0.0f;
#pragma unroll
  for (int s = 0; s < kSteps; ++s) {
    acc_new[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a0[s]),
                                                        __builtin_bit_cast(bf16x8, b[s]), acc_new[0], 0, 0, 0);
    acc_new[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a1[s]),
                                                        __builtin_bit_cast(bf16x8, b[s]), acc_new[1], 0, 0, 0);
#pragma unroll
    for (int e = s * kPer; e < (s + 1) * kPer; ++e) {
      const int t = e >> 4, r = e & 15;
      col[t][r] += __builtin_amdgcn_exp2f(__builtin_fmaf(acc_old[t][r], c, -ref));
    }
  }
#pragma unroll
  for (int s = 0; s < kSteps; ++s) {
    __builtin_amdgcn_sched_group_barrier(kSchedMfma, 1, 0);
    __builtin_amdgcn_sched_group_barrier(kSchedValu, 3 * kPer / 2, 0);
    __builtin_amdgcn_sched_group_barrier(kSchedMfma, 1, 0);
    __builtin_amdgcn_sched_group_barrier(kSchedValu, 3 * kPer / 2, 0);
  }
}

// operands: at least kThreads * kSteps * 3 * 16 bytes of bf16 values.  out: gridDim.x * kThreads floats.
__global__ __launch_bounds__(kThreads, 2) void mix_ceiling_kernel(const u32x4* __restrict__ operands, int iters, float c,
                                                                  float ref, float* __restrict__ out) {
  u32x4 a0[kSteps], a1[kSteps], b[kSteps];
#pragma unroll
  for (int s = 0; s < kSteps; ++s) {
    a0[s] = operands[(3 * s) * kThreads + threadIdx.x];
    a1[s] = operands[(3 * s + 1) * kThreads + threadIdx.x];
    b[s] = operands[(3 * s + 2) * kThreads + threadIdx.x];
  }
  f32x16 acc0[2], acc1[2], col[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc0[t][r] = acc1[t][r] = col[t][r] = 0.0f;
  for (int it = 0; it < iters; ++it) {
    mix_half(acc1, acc0, col, a0, a1, b, c, ref);
    mix_half(acc0, acc1, col, a0, a1, b, c, ref);
  }
  float v = 0.0f;
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) v += col[t][r] + acc0[t][r];
  out[(size_t)blockIdx.x * kThreads + threadIdx.x] = v;
}

}  // namespace

// Enqueues one launch on `hip_stream`.  operands: device, >= kvcrush_bench_mix_operand_bytes() bytes
// of bf16 values; out: device, grid * 256 floats.  Returns the matrix floating-point operations of the
// launch (the vector work is overhead, as it is in the score kernels); 0 on a bad argument or a refused launch.
extern "C" double kvcrush_bench_mix_ceiling(const void* operands, int32_t iters, int32_t grid, float* out,
                                            void* hip_stream) {
  if (!operands || !out || iters < 1 || grid < 1) return 0.0;
  // scale as at D = 128; the reference keeps every exponential finite and non-zero
  hipLaunchKernelGGL(mix_ceiling_kernel, dim3((unsigned)grid), dim3(kThreads), 0, (hipStream_t)hip_stream,
                     (const u32x4*)operands, iters, 0.12752f, 4.0f, out);
  if (hipGetLastError() != hipSuccess) return 0.0;
  return (double)grid * (kThreads / 64) * (double)iters * (2 * 2 * kSteps) * (2.0 * 32 * 32 * 16);
}

extern "C" size_t kvcrush_bench_mix_operand_bytes(void) { return (size_t)kThreads * kSteps * 3 * sizeof(u32x4); }
