// Decoding-time update of the running scores (KVCrush Sec. 1: the cache grows
// by one entry per generated token; the H2O importance the method builds on,
// Sec. 2.3, keeps accumulating the attention every cached token receives).
//
// One call = one new token per sequence: its query of every head attends to
// the S cached keys and the resulting probability row is added to the scores.
// A matrix-vector product per head: HBM-bound on reading K once
// (B*Hkv*S*D*sizeof bytes); the exponentials and the fp32 dot products are far
// below the VALU's rate at that pace.
//
//   append_logits_kernel   workgroup = 256 keys of one KV head.  A key row is
//                          read as 16-byte vectors by neighbouring lanes (whole
//                          cache lines per wave instruction); the queries of up
//                          to 8 heads of the KV group sit in registers, so K is
//                          read once for the group.  Leaves base-2 logits in the
//                          workspace and one (max, sum) pair per workgroup, head.
//   append_update_kernel   merges the pairs into the row normaliser, turns
//                          logits into probabilities, sums the group's heads in
//                          ascending order and updates the score row.
#include <cmath>

#include "common.h"

namespace {

typedef uint32_t vec16 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / KVC_WAVE;
constexpr int kKeysPerWg = 256;
constexpr int kHeadChunk = 8;  // query heads whose vectors are held in registers at once
constexpr float kNegBig = -1.0e30f;

struct AppendParams {
  const char* q_new;   // [B,Hq,D]
  const char* k;       // [B,Hkv,capacity,D]
  float* scores;       // [B,Hs,capacity]
  float* logits;       // workspace [B,Hq,S]
  float2* part;        // workspace [B,Hq,n_kb]
  int B, Hq, Hkv, S, capacity, G, reduce_groups, n_kb;
  float scale_log2;    // log2(e) / sqrt(D)
};

template <bool BF16>
__device__ __forceinline__ void unpack(const vec16& x, float (&f)[BF16 ? 8 : 4]) {
  if constexpr (BF16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(x[i] << 16);
      f[2 * i + 1] = __uint_as_float(x[i] & 0xFFFF0000u);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) f[i] = __uint_as_float(x[i]);
  }
}

__device__ __forceinline__ float block_max(float v, float* red) {
#pragma unroll
  for (int off = KVC_WAVE / 2; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  __syncthreads();  // `red` may still be read from the previous use
  if (kvc::lane_id() == 0) red[threadIdx.x / KVC_WAVE] = v;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) r = fmaxf(r, red[w]);
  return r;
}

__device__ __forceinline__ float block_sum(float v, float* red) {
#pragma unroll
  for (int off = KVC_WAVE / 2; off > 0; off >>= 1) v += __shfl_xor(v, off);
  __syncthreads();
  if (kvc::lane_id() == 0) red[threadIdx.x / KVC_WAVE] = v;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) r += red[w];
  return r;
}

template <bool BF16, int D>
__global__ __launch_bounds__(kThreads) void append_logits_kernel(AppendParams p) {
  constexpr int kRowBytes = D * (BF16 ? 2 : 4);
  constexpr int kLanesPerRow = kRowBytes / 16;          // 8, 16 or 32
  constexpr int kRowsPerWave = KVC_WAVE / kLanesPerRow;  // rows covered by one wave load
  constexpr int kElems = BF16 ? 8 : 4;                   // values per 16-byte vector
  constexpr int kIters = (kKeysPerWg / kWaves) / kRowsPerWave;
  constexpr int kUnroll = 4;
  static_assert(kIters % kUnroll == 0, "unroll must divide the trip count");

  __shared__ float lds_logit[kHeadChunk][kKeysPerWg];
  __shared__ float red[kWaves];

  const int tid = threadIdx.x, lane = kvc::lane_id(), wave = tid / KVC_WAVE;
  const int kb = blockIdx.x, bg = blockIdx.y;  // bg = b * Hkv + kv head
  const int b = bg / p.Hkv, g = bg % p.Hkv;
  const int S = p.S;
  const int k0 = kb * kKeysPerWg;
  const int col = lane % kLanesPerRow, sub = lane / kLanesPerRow;
  const char* kh = p.k + (size_t)bg * p.capacity * kRowBytes;

  for (int h0 = 0; h0 < p.G; h0 += kHeadChunk) {
    const int nh = min(kHeadChunk, p.G - h0);
    // this lane's slice of every query vector of the chunk
    float qv[kHeadChunk][kElems];
#pragma unroll
    for (int i = 0; i < kHeadChunk; ++i) {
      const int h = g * p.G + h0 + min(i, nh - 1);
      const vec16 x = *(const vec16*)(p.q_new + ((size_t)b * p.Hq + h) * kRowBytes + col * 16);
      unpack<BF16>(x, qv[i]);
    }
    for (int it0 = 0; it0 < kIters; it0 += kUnroll) {
      vec16 kx[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int key = k0 + wave * (kKeysPerWg / kWaves) + (it0 + u) * kRowsPerWave + sub;
        kx[u] = *(const vec16*)(kh + (size_t)min(key, S - 1) * kRowBytes + col * 16);
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        float kf[kElems];
        unpack<BF16>(kx[u], kf);
        const int lk = wave * (kKeysPerWg / kWaves) + (it0 + u) * kRowsPerWave + sub;
#pragma unroll
        for (int i = 0; i < kHeadChunk; ++i) {
          if (i < nh) {  // uniform
            float d = 0.0f;
#pragma unroll
            for (int e = 0; e < kElems; ++e) d = __builtin_fmaf(kf[e], qv[i][e], d);
#pragma unroll
            for (int off = kLanesPerRow / 2; off > 0; off >>= 1) d += __shfl_xor(d, off);
            if (col == 0) lds_logit[i][lk] = d * p.scale_log2;
          }
        }
      }
    }
    __syncthreads();
    // one key per thread: logits out (coalesced), block (max, sum of 2^(x - max)) per head
    const int key = k0 + tid;
    for (int i = 0; i < nh; ++i) {
      const int h = g * p.G + h0 + i;
      const float x = key < S ? lds_logit[i][tid] : kNegBig;
      if (key < S) p.logits[((size_t)b * p.Hq + h) * S + key] = x;
      const float m = block_max(x, red);
      const float l = block_sum(key < S ? __builtin_amdgcn_exp2f(x - m) : 0.0f, red);
      if (tid == 0) p.part[((size_t)b * p.Hq + h) * p.n_kb + kb] = make_float2(m, l);
    }
    __syncthreads();  // lds_logit is rewritten by the next chunk of heads
  }
}

__global__ __launch_bounds__(kThreads) void append_update_kernel(AppendParams p) {
  __shared__ float red[kWaves];
  const int tid = threadIdx.x;
  const int kb = blockIdx.x, row = blockIdx.y;  // row = b * Hs + r
  const int Hs = p.reduce_groups ? p.Hkv : p.Hq;
  const int b = row / Hs, r = row % Hs;
  const int h_first = p.reduce_groups ? r * p.G : r, n_heads = p.reduce_groups ? p.G : 1;
  const int key = kb * kKeysPerWg + tid;
  float acc = 0.0f;
  for (int i = 0; i < n_heads; ++i) {
    const size_t bh = (size_t)b * p.Hq + h_first + i;
    // row normaliser from the per-workgroup pairs
    float m = kNegBig;
    for (int j = tid; j < p.n_kb; j += kThreads) m = fmaxf(m, p.part[bh * p.n_kb + j].x);
    m = block_max(m, red);
    float l = 0.0f;
    for (int j = tid; j < p.n_kb; j += kThreads) {
      const float2 ml = p.part[bh * p.n_kb + j];
      l += ml.y * __builtin_amdgcn_exp2f(ml.x - m);
    }
    l = block_sum(l, red);
    const float lse2 = m + __builtin_amdgcn_logf(l);
    if (key < p.S) acc += __builtin_amdgcn_exp2f(p.logits[bh * p.S + key] - lse2);
  }
  if (key < p.S) {
    float* dst = p.scores + (size_t)row * p.capacity + key;
    *dst = (key == p.S - 1 ? 0.0f : *dst) + acc;  // the new token's slot starts from nothing
  }
}

size_t logits_bytes(const kvcrush_shape* s) {
  return kvc::align_up((size_t)s->B * s->Hq * s->S * sizeof(float), 256);
}

int key_blocks(const kvcrush_shape* s) { return (s->S + kKeysPerWg - 1) / kKeysPerWg; }

size_t part_bytes(const kvcrush_shape* s) {
  return kvc::align_up((size_t)s->B * s->Hq * key_blocks(s) * sizeof(float2), 256);
}

bool append_shape_ok(const kvcrush_shape* s, int capacity) {
  if (!s) return false;
  if (s->B < 1 || s->Hq < 1 || s->Hkv < 1 || s->S < 1 || s->D < 1 || capacity < s->S) return false;
  if (s->Hq % s->Hkv != 0) return false;
  if (s->dtype != KVCRUSH_F32 && s->dtype != KVCRUSH_BF16) return false;
  if (s->reduce_groups != 0 && s->reduce_groups != 1) return false;
  if (s->obs_window != 0) return false;
  return true;
}

template <bool BF16, int D>
kvcrush_status launch_append(const AppendParams& p, hipStream_t stream) {
  hipLaunchKernelGGL((append_logits_kernel<BF16, D>), dim3(p.n_kb, p.B * p.Hkv), dim3(kThreads), 0, stream, p);
  if (kvc::launch_status() != KVCRUSH_OK) return KVCRUSH_ERR_HIP;
  const int Hs = p.reduce_groups ? p.Hkv : p.Hq;
  hipLaunchKernelGGL(append_update_kernel, dim3(p.n_kb, p.B * Hs), dim3(kThreads), 0, stream, p);
  return kvc::launch_status();
}

}  // namespace

extern "C" size_t kvcrush_scores_append_workspace(const kvcrush_shape* shape, int32_t capacity) {
  if (!append_shape_ok(shape, capacity)) return 0;
  return logits_bytes(shape) + part_bytes(shape);
}

extern "C" kvcrush_status kvcrush_scores_append(const kvcrush_shape* shape, int32_t capacity,
                                                const void* q_new, const void* k, float* scores,
                                                void* workspace, size_t workspace_bytes,
                                                void* hip_stream) {
  if (!append_shape_ok(shape, capacity)) return KVCRUSH_ERR_INVALID_ARG;
  if (shape->D != 64 && shape->D != 128) return KVCRUSH_ERR_UNSUPPORTED;
  if ((long long)shape->B * shape->Hq > 65535) return KVCRUSH_ERR_UNSUPPORTED;
  if (!q_new || !k || !scores) return KVCRUSH_ERR_INVALID_ARG;
  if (!kvc::aligned16(q_new) || !kvc::aligned16(k) || !kvc::aligned16(scores))
    return KVCRUSH_ERR_INVALID_ARG;
  if (!workspace || !kvc::aligned16(workspace) ||
      workspace_bytes < logits_bytes(shape) + part_bytes(shape))
    return KVCRUSH_ERR_WORKSPACE;
  AppendParams p;
  p.q_new = (const char*)q_new;
  p.k = (const char*)k;
  p.scores = scores;
  p.logits = (float*)workspace;
  p.part = (float2*)((char*)workspace + logits_bytes(shape));
  p.B = shape->B;
  p.Hq = shape->Hq;
  p.Hkv = shape->Hkv;
  p.S = shape->S;
  p.capacity = capacity;
  p.G = shape->Hq / shape->Hkv;
  p.reduce_groups = shape->reduce_groups;
  p.n_kb = key_blocks(shape);
  p.scale_log2 = (float)(1.4426950408889634 / sqrt((double)shape->D));
  hipStream_t stream = (hipStream_t)hip_stream;
  const bool bf16 = shape->dtype == KVCRUSH_BF16;
  if (bf16 && shape->D == 128) return launch_append<true, 128>(p, stream);
  if (bf16 && shape->D == 64) return launch_append<true, 64>(p, stream);
  if (!bf16 && shape->D == 128) return launch_append<false, 128>(p, stream);
  return launch_append<false, 64>(p, stream);
}
