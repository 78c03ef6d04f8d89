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
  // running scores moved along with the rows (decoding-time eviction), or null
  const float* scores;         // [B, Hs, S]
  float* scores_out;           // [B, Hs, dst_tokens]
  int Hkv, Hs, S, budget;      // S = tokens per head in the dense source (its stride)
  int dst_tokens;              // tokens per head in the destination (its stride), >= budget
  int vec_per_row;             // D*sizeof / 16
  int lanes_per_row;           // min(vec_per_row, workgroup size)
  int lane_shift;              // log2(lanes_per_row) if it is a power of two, else -1
  int block_size, blocks_per_seq;
  int block_shift;             // log2(block_size) if it is a power of two, else -1
};

constexpr int kCompactThreads = 256;

// Grid: x = blocks of retained tokens, y = KV head (then, behind the heads, score rows),
// z = sequence.  A workgroup moves kRowsInFlight groups of 256 / lanes_per_row rows; a lane's
// place in its row is fixed, so all index arithmetic is shifts, adds and one retained-index
// load per row: no division per vector.
// kRowsInFlight = independent 16-byte loads per lane and tensor.  The gather is one dependent
// chain (index, row, store) per lane, so a small problem finishes soonest when every row has a
// lane of its own and the whole transfer is in flight at once (1); from some tens of MiB on,
// fewer and longer-lived workgroups keep the memory system fuller (8).
template <int kRowsInFlight>
__global__ __launch_bounds__(kCompactThreads) void compact_kernel(CompactParams p) {
  const int tid = threadIdx.x, b = blockIdx.z;
  const int32_t* __restrict__ idx = p.idx + (size_t)b * p.budget;
  const int rows_per_group = kCompactThreads / p.lanes_per_row;  // (>= 1; lanes beyond the last whole row idle)
  const int span = rows_per_group * kRowsInFlight;                // retained tokens per workgroup
  if ((int)blockIdx.y >= p.Hkv) {
    // a score row: the running scores of this workgroup's retained tokens
    const int r = blockIdx.y - p.Hkv;
    const float* __restrict__ src = p.scores + ((size_t)b * p.Hs + r) * p.S;
    float* __restrict__ dst = p.scores_out + ((size_t)b * p.Hs + r) * p.dst_tokens;
    const int j_end = min(p.budget, ((int)blockIdx.x + 1) * span);
    for (int j = blockIdx.x * span + tid; j < j_end; j += kCompactThreads)
      dst[j] = src[min(max(idx[j], 0), p.S - 1)];
    return;
  }
  const int h = blockIdx.y;
  int r_in, vec0;
  if (p.lane_shift >= 0) {
    r_in = tid >> p.lane_shift;
    vec0 = tid & (p.lanes_per_row - 1);
  } else {
    r_in = tid / p.lanes_per_row;
    vec0 = tid - r_in * p.lanes_per_row;
  }
  const int j0 = blockIdx.x * span + r_in;
  const bool lane_used = r_in < rows_per_group;
  const size_t bh = (size_t)b * p.Hkv + h;
  for (int vec = vec0; vec < p.vec_per_row; vec += p.lanes_per_row) {  // (one trip unless a row is wider than 4 KiB)
    vec16 kv[kRowsInFlight], vv[kRowsInFlight];
    bool live[kRowsInFlight];
#pragma unroll
    for (int u = 0; u < kRowsInFlight; ++u) {
      const int j = j0 + u * rows_per_group;
      live[u] = lane_used && j < p.budget;
      if (live[u]) {
        // an index outside the sequence (a caller's mistake) is pulled inside rather than followed
        const int t = min(max(idx[j], 0), p.S - 1);
        size_t src_row;
        if (p.block_table) {
          int lb, off;
          if (p.block_shift >= 0) {
            lb = t >> p.block_shift;
            off = t & (p.block_size - 1);
          } else {
            lb = t / p.block_size;
            off = t - lb * p.block_size;
          }
          const size_t blk = (size_t)p.block_table[(size_t)b * p.blocks_per_seq + lb];
          src_row = (blk * p.block_size + off) * p.Hkv + h;
        } else {
          src_row = bh * p.S + t;
        }
        const size_t src = src_row * p.vec_per_row + vec;
        kv[u] = __builtin_nontemporal_load(p.k + src);
        vv[u] = __builtin_nontemporal_load(p.v + src);
      }
    }
#pragma unroll
    for (int u = 0; u < kRowsInFlight; ++u) {
      if (live[u]) {
        const size_t dst = (bh * p.dst_tokens + (j0 + u * rows_per_group)) * p.vec_per_row + vec;
        __builtin_nontemporal_store(kv[u], p.k_out + dst);
        __builtin_nontemporal_store(vv[u], p.v_out + dst);
      }
    }
  }
}

int log2_if_pow2(int x) {
  if (x <= 0 || (x & (x - 1)) != 0) return -1;
  int s = 0;
  while ((1 << s) < x) ++s;
  return s;
}

kvcrush_status launch_compact(CompactParams p, int B, hipStream_t stream) {
  p.lanes_per_row = std::min(p.vec_per_row, kCompactThreads);
  p.lane_shift = log2_if_pow2(p.lanes_per_row);
  p.block_shift = log2_if_pow2(p.block_size);
  const size_t moved = (size_t)4 * B * p.Hkv * p.budget * p.vec_per_row * 16;  // K and V, read and written
  const int in_flight = moved >= ((size_t)64 << 20) ? 8 : 1;
  const int rows_per_wg = (kCompactThreads / p.lanes_per_row) * in_flight;
  const long long gx = ((long long)p.budget + rows_per_wg - 1) / rows_per_wg;
  const int gy = p.Hkv + (p.scores ? p.Hs : 0);
  if (gx > 0x7FFFFFFFll || gy > 65535 || B > 65535) return KVCRUSH_ERR_UNSUPPORTED;
  const dim3 grid((unsigned)gx, (unsigned)gy, (unsigned)B);
  return in_flight == 8 ? kvc::launch(compact_kernel<8>, grid, dim3(kCompactThreads), 0, stream, p)
                        : kvc::launch(compact_kernel<1>, grid, dim3(kCompactThreads), 0, stream, p);
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
  p.scores = nullptr;
  p.scores_out = nullptr;
  p.Hkv = Hkv;
  p.Hs = 0;
  p.S = S;
  p.budget = budget;
  p.dst_tokens = budget;
  p.vec_per_row = (int)(row_bytes / 16);
  p.block_size = block_table ? block_size : 1;
  p.blocks_per_seq = block_table ? S / block_size : 0;
  return launch_compact(p, B, (hipStream_t)hip_stream);
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
  return kvc::launch(block_table_gather_kernel, dim3(gx, B), dim3(kCompactThreads), 0,
                     (hipStream_t)hip_stream, idx, block_table, block_table_out, budget, block_size,
                     S / block_size);
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

  CompactParams p;
  p.k = (const vec16*)k;
  p.v = (const vec16*)v;
  p.k_out = (vec16*)k_out;
  p.v_out = (vec16*)v_out;
  p.idx = idx;
  p.block_table = nullptr;
  p.scores = scores;
  p.scores_out = scores_out;
  p.Hkv = Hkv;
  p.Hs = Hs;
  p.S = cap_src;
  p.budget = budget;
  p.dst_tokens = cap_dst;
  p.vec_per_row = (int)(row_bytes / 16);
  p.block_size = 1;
  p.blocks_per_seq = 0;
  return launch_compact(p, B, (hipStream_t)hip_stream);  // K, V and the score rows in one launch
}
