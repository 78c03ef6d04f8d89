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
//   append_logits_mfma_kernel  (bf16 / fp16) workgroup = 256 keys of one KV head
//                          (dense cache or paged pool): four
//                          64-row K tiles go global -> LDS asynchronously, each
//                          wave multiplies its tile with the query vectors of
//                          the KV group's heads (the 32 columns of a 32x32x16
//                          MFMA; unused columns are zero), so K is read once for
//                          the whole group and the dot products cost the VALU
//                          nothing.  Leaves base-2 logits in the workspace and
//                          one (max, sum) pair per workgroup and head.
//   append_logits_kernel   (fp32 inputs) the same on the VALU: a key row is read
//                          as 16-byte vectors by neighbouring lanes, the queries
//                          of up to 8 heads sit in registers.
//   append_update_kernel   merges the pairs into the row normaliser, turns
//                          logits into probabilities, sums the group's heads in
//                          ascending order and updates the score row.
#include <cmath>

#include "common.h"
#include "tiles.h"

namespace {

using namespace kvc::tiles;  // kThreads = 256, kWaves = 4, kNegBig, tile helpers

typedef uint32_t vec16 __attribute__((ext_vector_type(4)));

constexpr int kKeysPerWg = 256;
constexpr int kHeadChunk = 8;  // VALU path: query heads whose vectors are held in registers at once

struct AppendParams {
  const char* q_new;   // [B,Hq,D]
  const char* k;       // [B,Hkv,capacity,D]
  float* scores;       // [B,Hs,capacity]
  float* logits;       // workspace [B,Hq,S]
  float2* part;        // workspace [B,Hq,n_kb]
  const int* lengths;  // null, or [B]: valid tokens of each sequence (<= S), read on the device
  const int* block_table;  // null: k is dense [B,Hkv,capacity,D]; else k is a pool
                           // [n_blocks,block_size,Hkv,D] and block_table [B,capacity/block_size]
  int block_size;
  int B, Hq, Hkv, S, capacity, G, reduce_groups;  // S: valid tokens, or their upper bound with lengths
  int logit_keys, n_kb;  // keys per workgroup of the logits kernel, and how many such blocks S has
  float scale_log2;    // log2(e) x softmax scale (1 / sqrt(D) unless the caller set one)
};

// First byte of key row `key` of sequence b, KV head g (bg = b * Hkv + g).
__device__ __forceinline__ const char* key_row(const AppendParams& p, int b, int g, int bg, int key,
                                               int row_bytes) {
  if (!p.block_table) return p.k + ((size_t)bg * p.capacity + key) * row_bytes;
  const int blk = p.block_table[(size_t)b * (p.capacity / p.block_size) + key / p.block_size];
  return p.k + (((size_t)blk * p.block_size + key % p.block_size) * p.Hkv + g) * row_bytes;
}

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
  const int S = p.lengths ? min(max(p.lengths[b], 1), p.S) : p.S;
  const int k0 = kb * kKeysPerWg;
  if (k0 >= S) return;  // this sequence is shorter than the launch's upper bound (uniform exit)
  const int col = lane % kLanesPerRow, sub = lane / kLanesPerRow;

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
        kx[u] = *(const vec16*)(key_row(p, b, g, bg, min(key, S - 1), kRowBytes) + col * 16);
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
      if (key < S) p.logits[((size_t)b * p.Hq + h) * p.S + key] = x;
      const float m = block_max(x, red);
      const float l = block_sum(key < S ? __builtin_amdgcn_exp2f(x - m) : 0.0f, red);
      if (tid == 0) p.part[((size_t)b * p.Hq + h) * p.n_kb + kb] = make_float2(m, l);
    }
    __syncthreads();  // lds_logit is rewritten by the next chunk of heads
  }
}

// bf16: logits of 256 keys x up to 32 heads per pass on the matrix cores.
// TPW: 64-row tiles per workgroup (4: one tile per wave; 2: two waves share a tile, one 32-row half
// each, which halves the LDS per workgroup so that more of them overlap their loads on a CU).
template <int D, int TPW, bool F16>
__global__ __launch_bounds__(kThreads) void append_logits_mfma_kernel(AppendParams p) {
  using C = Cfg<true, D>;
  constexpr int kSubs = 2 * TPW / kWaves;  // 32-row halves a wave multiplies: 2 or 1
  __shared__ __attribute__((aligned(1024))) char lds[TPW][C::kTileBytes];
  __shared__ float red[2][kWaves][32];

  const int tid = threadIdx.x, lane = kvc::lane_id(), wave = tid / KVC_WAVE;
  const int kb = blockIdx.x, bg = blockIdx.y;  // bg = b * Hkv + kv head
  const int b = bg / p.Hkv, g = bg % p.Hkv;
  const int S = p.lengths ? min(max(p.lengths[b], 1), p.S) : p.S;
  const int k0 = kb * (C::kTile * TPW);
  if (k0 >= S) return;  // this sequence is shorter than the launch's upper bound (uniform exit)
  const char* kh = p.k + (size_t)bg * p.capacity * C::kRowBytes;

  uint32_t rel[C::kLoadsPerWave];
  tile_lane_offsets<C>(rel, wave, lane);
#pragma unroll
  for (int w = 0; w < TPW; ++w) {
    const int row0 = k0 + C::kTile * w;
    if (row0 >= S) continue;  // tiles past the end stay unread
    if (!p.block_table) {
      tile_load_async<C>(kh, row0, S, lds[w], rel, wave, lane);
    } else {
      // paged pool: the same LDS image, every 16-byte chunk fetched from its row's block
#pragma unroll
      for (int j = 0; j < C::kLoadsPerWave; ++j) {
        int row, chunk;
        tile_lane_chunk<C>(wave, lane, j, row, chunk);
        const int in_row = chunk * 16;
        const char* src = key_row(p, b, g, bg, min(row0 + row, S - 1), C::kRowBytes) + in_row;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)(lds[w] + (wave + kWaves * j) * 1024),
                                         16, 0, 0);
      }
    }
  }
  const int n = lane & 31;  // result column of this lane = head inside the chunk
  // query vectors of a chunk of up to 32 heads, as the MFMA's column operand (issued before the
  // wait for the tiles, so that the two latencies overlap)
  u32x4 qf[C::kSteps];
  auto load_q = [&](int h0) {
    const int nh = min(32, p.G - h0);
    const size_t bh = (size_t)b * p.Hq + g * p.G + h0 + min(n, nh - 1);
#pragma unroll
    for (int s = 0; s < C::kSteps; ++s) {
      u32x4 v = *(const u32x4*)(p.q_new + bh * C::kRowBytes + (s + (lane >> 5) * C::kSteps) * 16);
      if (n >= nh) v = u32x4{0u, 0u, 0u, 0u};
      qf[s] = v;
    }
  };
  load_q(0);
  wait_async_loads();
  __syncthreads();

  const int off0 = lds_frag_offset0<C>(lane);
  const int my_tile = wave % TPW, sub0 = (wave / TPW) * kSubs;  // this wave's rows: tile, first half
  const int key_base = k0 + C::kTile * my_tile + 32 * sub0 + 4 * (lane >> 5);  // + 32 * sub + 8 * (r / 4) + r % 4
  for (int h0 = 0; h0 < p.G; h0 += 32) {
    const int nh = min(32, p.G - h0);
    const size_t bh = (size_t)b * p.Hq + g * p.G + h0 + min(n, nh - 1);
    if (h0 > 0) load_q(h0);
    f32x16 acc[kSubs];
#pragma unroll
    for (int sub = 0; sub < kSubs; ++sub) {
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[sub][r] = 0.0f;
#pragma unroll
      for (int s = 0; s < C::kSteps; ++s)
        mma_step<true, F16>(acc[sub], lds_frag<C>(lds[my_tile], off0, sub0 + sub, s), qf[s]);
    }
    // this lane: 16 * kSubs keys of head n.  Keys past the end (and whole unread tiles) are masked here.
    float m = kNegBig;
#pragma unroll
    for (int sub = 0; sub < kSubs; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = key_base + 32 * sub + 8 * (r >> 2) + (r & 3);
        const float x = key < S ? acc[sub][r] * p.scale_log2 : kNegBig;
        acc[sub][r] = x;
        m = fmaxf(m, x);
      }
    m = fmaxf(m, __shfl_xor(m, 32));
    if (lane < 32) red[0][wave][n] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0][0][n], red[0][1][n]), fmaxf(red[0][2][n], red[0][3][n]));
    float l = 0.0f;
#pragma unroll
    for (int sub = 0; sub < kSubs; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) l += __builtin_amdgcn_exp2f(acc[sub][r] - m);  // masked keys: 2^-huge = 0
    l += __shfl_xor(l, 32);
    if (lane < 32) red[1][wave][n] = l;
    __syncthreads();
    if (tid < nh) {
      const float lt = (red[1][0][tid] + red[1][1][tid]) + (red[1][2][tid] + red[1][3][tid]);
      p.part[((size_t)b * p.Hq + g * p.G + h0 + tid) * p.n_kb + kb] = make_float2(m, lt);
    }
    if (n < nh) {
      float* dst = p.logits + bh * p.S;
#pragma unroll
      for (int sub = 0; sub < kSubs; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = key_base + 32 * sub + 8 * (r >> 2) + (r & 3);
          if (key < S) dst[key] = acc[sub][r];
        }
    }
    __syncthreads();  // `red` is rewritten by the next chunk of heads
  }
}

__global__ __launch_bounds__(kThreads) void append_update_kernel(AppendParams p) {
  __shared__ float red[kWaves];
  const int tid = threadIdx.x;
  const int kb = blockIdx.x, row = blockIdx.y;  // row = b * Hs + r
  const int Hs = p.reduce_groups ? p.Hkv : p.Hq;
  const int b = row / Hs, r = row % Hs;
  const int h_first = p.reduce_groups ? r * p.G : r, n_heads = p.reduce_groups ? p.G : 1;
  const int S = p.lengths ? min(max(p.lengths[b], 1), p.S) : p.S;
  if (kb * kKeysPerWg >= S) return;
  const int n_kb = (S + p.logit_keys - 1) / p.logit_keys;  // blocks that wrote a pair for this sequence
  const int key = kb * kKeysPerWg + tid;
  float acc = 0.0f;
  for (int i = 0; i < n_heads; ++i) {
    const size_t bh = (size_t)b * p.Hq + h_first + i;
    // row normaliser from the per-workgroup pairs
    float m = kNegBig;
    for (int j = tid; j < n_kb; j += kThreads) m = fmaxf(m, p.part[bh * p.n_kb + j].x);
    m = block_max(m, red);
    float l = 0.0f;
    for (int j = tid; j < n_kb; j += kThreads) {
      const float2 ml = p.part[bh * p.n_kb + j];
      l += ml.y * __builtin_amdgcn_exp2f(ml.x - m);
    }
    l = block_sum(l, red);
    const float lse2 = m + __builtin_amdgcn_logf(l);
    if (key < S) acc += __builtin_amdgcn_exp2f(p.logits[bh * p.S + key] - lse2);
  }
  if (key < S) {
    float* dst = p.scores + (size_t)row * p.capacity + key;
    *dst = (key == S - 1 ? 0.0f : *dst) + acc;  // the new token's slot starts from nothing
  }
}

size_t logits_bytes(const kvcrush_shape* s) {
  return kvc::align_up((size_t)s->B * s->Hq * s->S * sizeof(float), 256);
}

// Keys per workgroup of the logits kernel.  (Two tiles per workgroup on the matrix-core path, 128 keys,
// measured no faster than four: the kernel is not short of loads in flight.)
constexpr int kMfmaTilesPerWg = 4;
int logit_keys(const kvcrush_shape* s) { return s->dtype != KVCRUSH_F32 ? 64 * kMfmaTilesPerWg : kKeysPerWg; }

int key_blocks(const kvcrush_shape* s) { return (s->S + logit_keys(s) - 1) / logit_keys(s); }

size_t part_bytes(const kvcrush_shape* s) {
  return kvc::align_up((size_t)s->B * s->Hq * key_blocks(s) * sizeof(float2), 256);
}

bool append_shape_ok(const kvcrush_shape* s, int capacity) {
  if (!s) return false;
  if (s->B < 1 || s->Hq < 1 || s->Hkv < 1 || s->S < 1 || s->D < 1 || capacity < s->S) return false;
  if (s->Hq % s->Hkv != 0) return false;
  if (s->dtype != KVCRUSH_F32 && s->dtype != KVCRUSH_BF16 && s->dtype != KVCRUSH_F16) return false;
  if (s->reduce_groups != 0 && s->reduce_groups != 1) return false;
  if (s->obs_window != 0) return false;
  if (!(s->softmax_scale >= 0.0f) || s->softmax_scale > 1.0e6f) return false;  // also rejects NaN
  return true;
}

template <bool BF16, int D, bool F16 = false>
kvcrush_status launch_append(const AppendParams& p, hipStream_t stream) {
  kvcrush_status st;
  if constexpr (BF16) {
    st = kvc::launch(append_logits_mfma_kernel<D, kMfmaTilesPerWg, F16>, dim3(p.n_kb, p.B * p.Hkv),
                       dim3(kThreads), 0, stream, p);
  } else {
    st = kvc::launch(append_logits_kernel<BF16, D>, dim3(p.n_kb, p.B * p.Hkv), dim3(kThreads), 0, stream, p);
  }
  if (st != KVCRUSH_OK) return st;
  const int Hs = p.reduce_groups ? p.Hkv : p.Hq;
  return kvc::launch(append_update_kernel, dim3((p.S + kKeysPerWg - 1) / kKeysPerWg, p.B * Hs), dim3(kThreads), 0,
                     stream, p);
}

}  // namespace

extern "C" size_t kvcrush_scores_append_workspace(const kvcrush_shape* shape, int32_t capacity) {
  if (!append_shape_ok(shape, capacity)) return 0;
  return logits_bytes(shape) + part_bytes(shape);
}

extern "C" kvcrush_status kvcrush_scores_append(const kvcrush_shape* shape, int32_t capacity,
                                                const int32_t* lengths, const void* q_new,
                                                const void* k, const int32_t* block_table,
                                                int32_t block_size, float* scores, void* workspace,
                                                size_t workspace_bytes, void* hip_stream) {
  if (!append_shape_ok(shape, capacity)) return KVCRUSH_ERR_INVALID_ARG;
  if (block_table && (block_size < 1 || capacity % block_size != 0)) return KVCRUSH_ERR_INVALID_ARG;
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
  p.lengths = lengths;
  p.block_table = block_table;
  p.block_size = block_table ? block_size : 1;
  p.B = shape->B;
  p.Hq = shape->Hq;
  p.Hkv = shape->Hkv;
  p.S = shape->S;
  p.capacity = capacity;
  p.G = shape->Hq / shape->Hkv;
  p.reduce_groups = shape->reduce_groups;
  p.logit_keys = logit_keys(shape);
  p.n_kb = key_blocks(shape);
  p.scale_log2 = (float)(1.4426950408889634 *
                         (shape->softmax_scale != 0.0f ? (double)shape->softmax_scale : 1.0 / sqrt((double)shape->D)));
  hipStream_t stream = (hipStream_t)hip_stream;
  if (shape->dtype == KVCRUSH_F16)
    return shape->D == 128 ? launch_append<true, 128, true>(p, stream) : launch_append<true, 64, true>(p, stream);
  const bool bf16 = shape->dtype == KVCRUSH_BF16;
  if (bf16 && shape->D == 128) return launch_append<true, 128>(p, stream);
  if (bf16 && shape->D == 64) return launch_append<true, 64>(p, stream);
  if (!bf16 && shape->D == 128) return launch_append<false, 128>(p, stream);
  return launch_append<false, 64>(p, stream);
}
