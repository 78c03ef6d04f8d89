// Stage 5: gather the retained K/V rows into the dense reduced cache
// (KVCrush Sec. 3.2: the retained tokens form the final cache).
//
// HBM-bound copy.  A token row of one head is D*sizeof bytes (256 B for
// D = 128 bf16) and is moved as 16-byte vectors: consecutive lanes take
// consecutive vectors of a row, consecutive rows follow in the same wave, so
// the stores are fully contiguous and each load touches whole 128-byte lines.
// idx is ascending, so the reads sweep the source forwards as well.
#include <algorithm>

#include "common.h"

namespace {

typedef uint32_t vec16 __attribute__((ext_vector_type(4)));  // one 16-byte vector

struct CompactParams {
  const vec16* k;
  const vec16* v;
  vec16* k_out;
  vec16* v_out;
  const int32_t* idx;
  const int32_t* block_table;  // null: dense source
  int B, Hkv, S, budget;       // S = tokens per head in the dense source (its stride)
  int dst_tokens;              // tokens per head in the destination (its stride), >= budget
  int vec_per_row;             // D*sizeof / 16
  int block_size, blocks_per_seq;
  long long total_vec;         // B*Hkv*budget*vec_per_row
};

constexpr int kCompactThreads = 256;
constexpr int kRowsInFlight = 4;  // independent 16-byte loads per lane and tensor

__global__ __launch_bounds__(kCompactThreads) void compact_kernel(CompactParams p) {
  const long long stride = (long long)gridDim.x * kCompactThreads;
  long long i0 = (long long)blockIdx.x * kCompactThreads + threadIdx.x;
  // Each lane owns kRowsInFlight vectors, `stride` apart, so that all their
  // loads are issued before the first store.
  for (; i0 < p.total_vec; i0 += stride * kRowsInFlight) {
    vec16 kv[kRowsInFlight], vv[kRowsInFlight];
    long long dst[kRowsInFlight];
#pragma unroll
    for (int u = 0; u < kRowsInFlight; ++u) {
      const long long i = i0 + (long long)u * stride;
      dst[u] = -1;
      if (i < p.total_vec) {
        const int vec = (int)(i % p.vec_per_row);
        const long long row = i / p.vec_per_row;      // (b*Hkv + h)*budget + j
        const int j = (int)(row % p.budget);
        const long long bh = row / p.budget;
        const int h = (int)(bh % p.Hkv);
        const int b = (int)(bh / p.Hkv);
        // an index outside the sequence (a caller's mistake) is pulled inside rather than followed
        const int t = min(max(p.idx[(long long)b * p.budget + j], 0), p.S - 1);
        long long src_row;
        if (p.block_table) {
          const long long blk = p.block_table[(long long)b * p.blocks_per_seq + t / p.block_size];
          src_row = (blk * p.block_size + t % p.block_size) * p.Hkv + h;
        } else {
          src_row = bh * p.S + t;
        }
        const long long src = src_row * p.vec_per_row + vec;
        kv[u] = __builtin_nontemporal_load(p.k + src);
        vv[u] = __builtin_nontemporal_load(p.v + src);
        dst[u] = (bh * p.dst_tokens + j) * p.vec_per_row + vec;
      }
    }
#pragma unroll
    for (int u = 0; u < kRowsInFlight; ++u) {
      if (dst[u] >= 0) {
        __builtin_nontemporal_store(kv[u], p.k_out + dst[u]);
        __builtin_nontemporal_store(vv[u], p.v_out + dst[u]);
      }
    }
  }
}

// Running scores of the kept tokens, moved with them (decoding-time eviction).
struct ScoreGatherParams {
  const float* scores;   // [rows_per_seq * B, cap_src]
  float* scores_out;     // [rows_per_seq * B, cap_dst]
  const int32_t* idx;    // [B, budget]
  int Hs, cap_src, cap_dst, budget;
};

__global__ __launch_bounds__(kCompactThreads) void score_gather_kernel(ScoreGatherParams p) {
  const int row = blockIdx.y;  // b * Hs + r
  const int b = row / p.Hs;
  for (int j = blockIdx.x * kCompactThreads + threadIdx.x; j < p.budget; j += gridDim.x * kCompactThreads)
    p.scores_out[(size_t)row * p.cap_dst + j] =
        p.scores[(size_t)row * p.cap_src + min(max(p.idx[(size_t)b * p.budget + j], 0), p.cap_src - 1)];
}

kvcrush_status launch_compact(const CompactParams& p, hipStream_t stream) {
  const long long per_block = (long long)kCompactThreads * kRowsInFlight;
  long long blocks = (p.total_vec + per_block - 1) / per_block;
  const long long max_blocks = 256 * 32;  // 256 CUs, several waves each; the rest grid-strides
  if (blocks > max_blocks) blocks = max_blocks;
  hipLaunchKernelGGL(compact_kernel, dim3((unsigned)blocks), dim3(kCompactThreads), 0, stream, p);
  return kvc::launch_status();
}

}  // namespace

extern "C" kvcrush_status kvcrush_compact(int32_t B, int32_t Hkv, int32_t S, int32_t D, int32_t dtype,
                                          int32_t budget, const void* k, const void* v,
                                          const int32_t* idx, const int32_t* block_table,
                                          int32_t block_size, void* k_out, void* v_out,
                                          void* hip_stream) {
  if (B < 1 || Hkv < 1 || S < 1 || D < 1 || budget < 0 || budget > S) return KVCRUSH_ERR_INVALID_ARG;
  if (dtype != KVCRUSH_F32 && dtype != KVCRUSH_BF16 && dtype != KVCRUSH_F16) return KVCRUSH_ERR_INVALID_ARG;
  const size_t row_bytes = (size_t)D * (dtype == KVCRUSH_F32 ? 4 : 2);
  if (row_bytes % 16 != 0) return KVCRUSH_ERR_UNSUPPORTED;
  if (block_table && (block_size < 1 || S % block_size != 0)) return KVCRUSH_ERR_INVALID_ARG;
  if (budget == 0) return KVCRUSH_OK;
  if (!k || !v || !idx || !k_out || !v_out) return KVCRUSH_ERR_INVALID_ARG;
  if (!kvc::aligned16(k) || !kvc::aligned16(v) || !kvc::aligned16(k_out) || !kvc::aligned16(v_out))
    return KVCRUSH_ERR_INVALID_ARG;

  CompactParams p;
  p.k = (const vec16*)k;
  p.v = (const vec16*)v;
  p.k_out = (vec16*)k_out;
  p.v_out = (vec16*)v_out;
  p.idx = idx;
  p.block_table = block_table;
  p.B = B;
  p.Hkv = Hkv;
  p.S = S;
  p.budget = budget;
  p.dst_tokens = budget;
  p.vec_per_row = (int)(row_bytes / 16);
  p.block_size = block_table ? block_size : 1;
  p.blocks_per_seq = block_table ? S / block_size : 0;
  p.total_vec = (long long)B * Hkv * budget * p.vec_per_row;

  return launch_compact(p, (hipStream_t)hip_stream);
}

// Page-level eviction on a paged pool whose block size is the selection unit: nothing moves, the
// reduced cache is the list of kept blocks.
__global__ __launch_bounds__(kCompactThreads) void block_table_gather_kernel(const int32_t* idx,
                                                                           const int32_t* block_table,
                                                                           int32_t* out, int budget,
                                                                           int unit, int blocks_src) {
  const int b = blockIdx.y, kept = budget / unit;
  for (int j = blockIdx.x * kCompactThreads + threadIdx.x; j < kept; j += gridDim.x * kCompactThreads)
    out[(size_t)b * kept + j] =
        block_table[(size_t)b * blocks_src + min(max(idx[(size_t)b * budget + (size_t)j * unit] / unit, 0), blocks_src - 1)];
}

extern "C" kvcrush_status kvcrush_compact_block_table(int32_t B, int32_t S, int32_t budget,
                                                      int32_t block_size, const int32_t* idx,
                                                      const int32_t* block_table,
                                                      int32_t* block_table_out, void* hip_stream) {
  if (B < 1 || S < 1 || block_size < 1 || budget < 0 || budget > S || S % block_size != 0 ||
      budget % block_size != 0)
    return KVCRUSH_ERR_INVALID_ARG;
  if (budget == 0) return KVCRUSH_OK;
  if (!idx || !block_table || !block_table_out) return KVCRUSH_ERR_INVALID_ARG;
  if (B > 65535) return KVCRUSH_ERR_UNSUPPORTED;
  const int kept = budget / block_size;
  const int gx = std::min(64, (kept + kCompactThreads - 1) / kCompactThreads);
  hipLaunchKernelGGL(block_table_gather_kernel, dim3(gx, B), dim3(kCompactThreads), 0,
                     (hipStream_t)hip_stream, idx, block_table, block_table_out, budget, block_size,
                     S / block_size);
  return kvc::launch_status();
}

extern "C" kvcrush_status kvcrush_compact_cache(int32_t B, int32_t Hkv, int32_t Hs, int32_t D,
                                                int32_t dtype, int32_t cap_src, int32_t cap_dst,
                                                int32_t budget, const void* k, const void* v,
                                                const float* scores, const int32_t* idx, void* k_out,
                                                void* v_out, float* scores_out, void* hip_stream) {
  if (B < 1 || Hkv < 1 || Hs < 1 || D < 1 || cap_src < 1 || cap_dst < 1 || budget < 0 ||
      budget > cap_src || budget > cap_dst)
    return KVCRUSH_ERR_INVALID_ARG;
  if (dtype != KVCRUSH_F32 && dtype != KVCRUSH_BF16 && dtype != KVCRUSH_F16) return KVCRUSH_ERR_INVALID_ARG;
  const size_t row_bytes = (size_t)D * (dtype == KVCRUSH_F32 ? 4 : 2);
  if (row_bytes % 16 != 0) return KVCRUSH_ERR_UNSUPPORTED;
  if (budget == 0) return KVCRUSH_OK;
  if (!k || !v || !idx || !k_out || !v_out || !scores || !scores_out) return KVCRUSH_ERR_INVALID_ARG;
  if (k == k_out || v == v_out || scores == scores_out) return KVCRUSH_ERR_INVALID_ARG;  // not in place
  if (!kvc::aligned16(k) || !kvc::aligned16(v) || !kvc::aligned16(k_out) || !kvc::aligned16(v_out))
    return KVCRUSH_ERR_INVALID_ARG;
  if ((long long)B * Hs > 65535) return KVCRUSH_ERR_UNSUPPORTED;

  CompactParams p;
  p.k = (const vec16*)k;
  p.v = (const vec16*)v;
  p.k_out = (vec16*)k_out;
  p.v_out = (vec16*)v_out;
  p.idx = idx;
  p.block_table = nullptr;
  p.B = B;
  p.Hkv = Hkv;
  p.S = cap_src;
  p.budget = budget;
  p.dst_tokens = cap_dst;
  p.vec_per_row = (int)(row_bytes / 16);
  p.block_size = 1;
  p.blocks_per_seq = 0;
  p.total_vec = (long long)B * Hkv * budget * p.vec_per_row;
  hipStream_t stream = (hipStream_t)hip_stream;
  if (launch_compact(p, stream) != KVCRUSH_OK) return KVCRUSH_ERR_HIP;

  ScoreGatherParams g;
  g.scores = scores;
  g.scores_out = scores_out;
  g.idx = idx;
  g.Hs = Hs;
  g.cap_src = cap_src;
  g.cap_dst = cap_dst;
  g.budget = budget;
  const int gx = std::min(64, (budget + kCompactThreads - 1) / kCompactThreads);
  hipLaunchKernelGGL(score_gather_kernel, dim3(gx, B * Hs), dim3(kCompactThreads), 0, stream, g);
  return kvc::launch_status();
}
