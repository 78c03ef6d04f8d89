// Stages 2-4 of the KVCrush step on gfx950: importance top-k, head-behaviour
// bit vectors (Alg. 1, Sec. 3.1), Hamming grouping and one representative per
// bucket (Alg. 2, Sec. 3.2), merged ascending index list.
//
// All integer / compare work on at most a few MiB, so the stage is bound by
// latency, not bandwidth: five short launches on one stream, no host round
// trip, no floating-point atomics (every tie is broken by token index, so the
// result is a pure function of the score tensor).
//
//   K1 topk_mask_kernel   one workgroup per (sequence, score row) plus one for
//                         the importance row: exact k-th largest by an MSB-first
//                         radix select (11 + 11 + 10 bits) over order-preserving
//                         integer keys held in LDS, then a 64-tokens-per-word
//                         bitmap of the selected set (ties: lowest index first).
//   K2 group_rank_kernel /  many small workgroups per sequence: pack the row
//      group_scatter_kernel bitmaps into per-token words, build the anchor,
//                         Hamming distance by xor+popcount, and a stable
//                         counting sort of the non-important tokens by distance
//                         (wave ballots give each token its rank among equal
//                         distances inside its wave; a small count table turns
//                         that into global ranks).
//   K3 medoid_kernel      one wavefront per bucket: per-head counts by ballot,
//                         integer cost, wave arg-min with token tie-break.
//   K4 emit_kernel        ordered compaction of (important | representative)
//                         bitmaps into the ascending index list.
//
// Variants on the same kernels.  Protected ends (Table 1's cache layout): the
// kernels are handed the tokens between the ends, K4 writes the ends around
// them.  Chunk- / page-level selection (Sec. 4.3.4, 4.3.5): K1's importance row
// ranks units (sums of their tokens' importances), K1b unit_rows_kernel turns the
// token bitmaps into per-unit rows (a unit's vector = its tokens' head vectors
// concatenated), K2-K4 then treat units as items; K2 and K3 are templates over
// the 64-bit words per vector (up to 16 = 1024 bits), with a workgroup-per-bucket
// K3 for the long vectors, whose buckets are few and large.
#include <algorithm>
#include <mutex>

#include "common.h"

namespace {

using kvc::lane_id;
using kvc::lanemask_lt;

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / KVC_WAVE;
constexpr int kMaxHs = 1024;  // bits per grouped item: score rows x tokens per unit
constexpr int kMaxW = kMaxHs / 64;

// Order-preserving map from fp32 to uint32 (larger float -> larger key);
// -0.0 is folded onto +0.0 so that the two compare equal, as they do as floats.
__device__ __forceinline__ uint32_t float_key(float x) {
  uint32_t u = __float_as_uint(x);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive moves (no LDS
// round trips): shifts by 1, 2, 4 and 8 lanes inside each row of 16 lanes (lanes shifted in
// from outside a row read zero), then lane 15 of rows 0 and 2 added to rows 1 and 3, then
// lane 31 added to rows 2 and 3.
__device__ __forceinline__ int wave_incl_scan(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);   // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);   // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);   // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);   // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1, 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2, 3
  return v;
}

__device__ __forceinline__ int wave_sum(int v) {
  return __builtin_amdgcn_readlane(wave_incl_scan(v), KVC_WAVE - 1);
}

// Lanes of the wave that hold the same small integer d (only `nbits` low bits
// can differ).  Invalid lanes get 0 and are in nobody's set.
__device__ __forceinline__ uint64_t match_peers(uint32_t d, int nbits, bool valid) {
  uint64_t peers = __ballot(valid);
  for (int b = 0; b < nbits; ++b) {
    const bool bit = (d >> b) & 1u;
    const uint64_t m = __ballot(bit);
    peers &= bit ? m : ~m;
  }
  return valid ? peers : 0ull;
}

// Chunk (64-token word) range owned by a wave when nw chunks are dealt out in
// contiguous runs, so that (wave, chunk, lane) order is token order.
__device__ __forceinline__ void wave_chunk_range(int nw, int nwaves, int wave, int& c0, int& c1) {
  const int per = (nw + nwaves - 1) / nwaves;
  c0 = min(nw, wave * per);
  c1 = min(nw, c0 + per);
}

// Words that one workgroup writes and another reads inside the same launch (row bitmaps,
// representative bitmaps) go through agent-scope accesses: such a store is written through to
// the point where all compute units see it, such a load is served from there.  (Full release /
// acquire fences would also do, but they write back and invalidate whole caches, tens of
// microseconds when every workgroup of a launch issues them.)
__device__ __forceinline__ void store_shared_word(uint64_t* p, uint64_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t load_shared_word(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Arrival of a workgroup at a counter that `expected` workgroups add to; true (for the whole
// workgroup) in the one that arrives last.  Every word that later readers need must have been
// written with store_shared_word (or an atomic): each thread waits here until its own vector
// memory operations have been acknowledged (vmcnt counts stores and atomics on this target),
// and only then does the workgroup's arrival become visible.  Contains barriers.
__device__ __forceinline__ bool arrive_last(uint32_t* counter, uint32_t expected, uint32_t* sh_flag) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0)
    *sh_flag = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == expected - 1u;
  __syncthreads();
  const bool last = *sh_flag != 0u;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  return last;
}

// ------------------------------------------------------------------ K1 ----
struct TopkParams {
  const float* scores;  // first selectable token of row 0 of sequence 0; rows are `ld` floats apart
  uint64_t* rowmask;    // [B,Hs+1,nw]; row Hs = important tokens
  uint32_t* keys_ws;    // [B,Hs+1,S] when the row does not fit LDS, else null
  int Hs, S, nw, kbit, n_important;  // S = selectable tokens per row (the middle, when ends are protected)
  int ld;               // row stride of `scores` in floats (the full sequence length)
  int unit;             // tokens per selection unit; the importance row then ranks S / unit units
  int importance_only;  // 1: no representatives and no bit words are wanted, the per-row masks are skipped
};

// Block-wide exclusive prefix sum of one int per thread, in thread order.
// `wave_tot` is LDS scratch of kSelWaves ints; contains two barriers.
__device__ __forceinline__ int block_excl_scan(int v, int* wave_tot) {
  const int lane = lane_id(), wave = threadIdx.x / KVC_WAVE, n_waves = blockDim.x / KVC_WAVE;
  const int incl = wave_incl_scan(v);
  if (lane == KVC_WAVE - 1) wave_tot[wave] = incl;
  __syncthreads();
  // (at most 16 waves: every wave scans the waves' totals itself, one per lane)
  const int tot_scan = wave_incl_scan(lane < n_waves ? wave_tot[lane] : 0);
  const int before = __shfl(tot_scan - (lane < n_waves ? wave_tot[lane] : 0), wave);
  __syncthreads();
  return before + incl - v;
}

constexpr int kRadixBins = 2048;  // 11 + 11 + 10 bits over three passes
constexpr int kBatch = 8;         // independent loads in flight per thread

// KEYS_IN_LDS: the row's keys live in the dynamic LDS buffer (the usual case);
// otherwise in the workspace.  Two instantiations rather than one generic
// pointer, so that the compiler knows LDS traffic cannot alias global traffic
// and keeps batches of loads in flight.
template <bool KEYS_IN_LDS>
__global__ __launch_bounds__(kSelThreads) void topk_mask_kernel(TopkParams p) {
  extern __shared__ uint32_t lds_keys[];
  __shared__ uint32_t hist[kRadixBins];
  __shared__ uint32_t sh_digit, sh_remaining, sh_count;
  __shared__ int wave_tot[kSelWaves];

  const int row = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x, lane = lane_id(), wave = tid / KVC_WAVE;
  const int Hs = p.Hs;
  // score rows rank tokens; the importance row ranks units of p.unit tokens (Sec. 4.3.5: a
  // page's importance is that of its tokens added up)
  const bool unit_row = row == Hs && p.unit > 1;
  const int S_tok = p.S;
  const int S = unit_row ? S_tok / p.unit : S_tok;
  const int nw = unit_row ? (S + 63) / 64 : p.nw;
  const int k = row < Hs ? p.kbit : p.n_important;
  uint64_t* __restrict__ mask_out = p.rowmask + ((size_t)b * (Hs + 1) + row) * p.nw;
  if (p.importance_only && row < Hs) return;  // (whole workgroup, before any barrier)

  if (k == 0 || k == S) {  // nothing or everything: no search needed
    for (int c = tid; c < nw; c += kSelThreads) {
      uint64_t w = 0;
      if (k == S) {
        const int rem = S - c * 64;
        w = rem >= 64 ? ~0ull : ((1ull << rem) - 1ull);
      }
      mask_out[c] = w;
    }
    return;
  }

  uint32_t* __restrict__ gkeys = KEYS_IN_LDS ? nullptr : p.keys_ws + ((size_t)b * (Hs + 1) + row) * p.S;
  auto key_at = [&](int t) -> uint32_t { return KEYS_IN_LDS ? lds_keys[t] : gkeys[t]; };
  auto key_put = [&](int t, uint32_t v) {
    if (KEYS_IN_LDS) lds_keys[t] = v; else gkeys[t] = v;
  };
  const float* __restrict__ sc = p.scores + (size_t)b * Hs * p.ld;
  const size_t ld = (size_t)p.ld;

  for (int i = tid; i < kRadixBins; i += kSelThreads) hist[i] = 0;
  // keys.  Rows that start on a 16-byte boundary are read four tokens a load (the importance row
  // moves Hs times a row's bytes through this one compute unit: wide loads are what it is bound by)
  int t_done = 0;
  if (((reinterpret_cast<uintptr_t>(sc) | (ld * sizeof(float))) & 15) == 0) {
    constexpr int kQuads = 2;  // independent quads per thread and row
    const int n4 = S_tok >> 2;
    for (int g0 = tid; g0 < n4; g0 += kQuads * kSelThreads) {
      float4 v[kQuads];
      auto quad = [&](int r, int u) {
        const int g = g0 + u * kSelThreads;
        return g < n4 ? *(const float4*)(sc + (size_t)r * ld + 4 * (size_t)g) : make_float4(0.f, 0.f, 0.f, 0.f);
      };
      if (row < Hs) {
#pragma unroll
        for (int u = 0; u < kQuads; ++u) v[u] = quad(row, u);
      } else {
#pragma unroll
        for (int u = 0; u < kQuads; ++u) v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        int r = 0;
        for (; r + 8 <= Hs; r += 8) {  // eight rows' loads in flight; the additions stay in row order
          float4 x[8][kQuads];
#pragma unroll
          for (int rr = 0; rr < 8; ++rr)
#pragma unroll
            for (int u = 0; u < kQuads; ++u) x[rr][u] = quad(r + rr, u);
#pragma unroll
          for (int rr = 0; rr < 8; ++rr)
#pragma unroll
            for (int u = 0; u < kQuads; ++u) {
              v[u].x = v[u].x + x[rr][u].x;
              v[u].y = v[u].y + x[rr][u].y;
              v[u].z = v[u].z + x[rr][u].z;
              v[u].w = v[u].w + x[rr][u].w;
            }
        }
        for (; r < Hs; ++r) {
#pragma unroll
          for (int u = 0; u < kQuads; ++u) {
            const float4 x = quad(r, u);
            v[u].x = v[u].x + x.x;
            v[u].y = v[u].y + x.y;
            v[u].z = v[u].z + x.z;
            v[u].w = v[u].w + x.w;
          }
        }
      }
#pragma unroll
      for (int u = 0; u < kQuads; ++u) {
        const int g = g0 + u * kSelThreads;
        if (g < n4) {
          const float e[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
          for (int j = 0; j < 4; ++j) key_put(4 * g + j, unit_row ? __float_as_uint(e[j]) : float_key(e[j]));
        }
      }
    }
    t_done = 4 * n4;
  }
  // the rest (or everything, for rows that are not aligned): kBatch tokens per thread at a time
  for (int t0 = t_done + tid; t0 < S_tok; t0 += kBatch * kSelThreads) {
    float v[kBatch];
    if (row < Hs) {
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int t = t0 + u * kSelThreads;
        v[u] = t < S_tok ? sc[(size_t)row * ld + t] : 0.0f;
      }
    } else {
      // token importance: fp32 sum of the score rows, taken in row order
#pragma unroll
      for (int u = 0; u < kBatch; ++u) v[u] = 0.0f;
      // eight rows' loads in flight at a time; the additions stay in row order
      int r = 0;
      for (; r + 8 <= Hs; r += 8) {
        float x[8][kBatch];
#pragma unroll
        for (int rr = 0; rr < 8; ++rr)
#pragma unroll
          for (int u = 0; u < kBatch; ++u) {
            const int t = t0 + u * kSelThreads;
            x[rr][u] = t < S_tok ? sc[(size_t)(r + rr) * ld + t] : 0.0f;
          }
#pragma unroll
        for (int rr = 0; rr < 8; ++rr)
#pragma unroll
          for (int u = 0; u < kBatch; ++u) v[u] = v[u] + x[rr][u];
      }
      for (; r < Hs; ++r) {
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
          const int t = t0 + u * kSelThreads;
          const float x = t < S_tok ? sc[(size_t)r * ld + t] : 0.0f;
          v[u] = v[u] + x;
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int t = t0 + u * kSelThreads;
      // (unit row: the token's importance itself is parked here, keys follow below)
      if (t < S_tok) key_put(t, unit_row ? __float_as_uint(v[u]) : float_key(v[u]));
    }
  }
  __syncthreads();
  if (unit_row) {
    // Unit importance = its tokens' importances added in token order.  Unit u reads slots
    // [u * unit, (u + 1) * unit) and its key goes to slot u; units are taken 1024 at a time,
    // reads and writes of a round apart, so a slot is never overwritten before its reader
    // (unit u / unit, which comes no later than unit u) has passed.
    for (int u0 = 0; u0 < S; u0 += kSelThreads) {
      const int u = u0 + tid;
      float acc = 0.0f;
      if (u < S)
        for (int j = 0; j < p.unit; ++j) acc = acc + __uint_as_float(key_at(u * p.unit + j));
      __syncthreads();
      if (u < S) key_put(u, float_key(acc));
      __syncthreads();
    }
  }

  // MSB-first radix select of the k-th largest key: 11, 11 and 10 bits a pass.
  // One LDS histogram shared by the workgroup; only keys that still match the
  // prefix found so far are counted, so passes two and three are nearly free.
  uint32_t prefix = 0, known = 0, remaining = (uint32_t)k;
#pragma unroll
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
    const int bins = pass == 2 ? 1024 : 2048;
    {
      // Counting the keys that still match the prefix (all of them in the first pass).  A wave
      // walks its own run of 64-token chunks and each lane keeps the bin of its previous counted
      // key with a count: keys 64 tokens apart are mostly of similar size, and equal keys share
      // every digit, so a lane adds to the histogram only when its bin changes (a few times, not
      // once per key).  If nearly the whole wave changes bin at nearly every key while sitting in
      // one bin (blocks of tokens alternating between sizes), those additions would hit one
      // address all at once and be served one by one: the wave then counts the rest of its keys
      // by ballot (the bin of the first lane left, one add of the popcount, three rounds at most).
      int pc0, pc1;
      wave_chunk_range(nw, kSelWaves, wave, pc0, pc1);
      uint32_t run_bin = 0, run_cnt = 0;
      bool by_ballot = false;  // wave-uniform
      for (int cb = pc0; cb < pc1; cb += 4) {
        uint32_t kk[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int t = (cb + u) * 64 + lane;
          kk[u] = (cb + u < pc1 && t < S) ? key_at(t) : 0u;
        }
        if (!by_ballot) {
          int changes = 0;
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int t = (cb + u) * 64 + lane;
            const uint32_t bin = (kk[u] >> shift) & (uint32_t)(bins - 1);
            if (cb + u < pc1 && t < S && (kk[u] & known) == prefix) {
              if (bin == run_bin) {
                ++run_cnt;
              } else {
                if (run_cnt) atomicAdd(&hist[run_bin], run_cnt);
                run_bin = bin;
                run_cnt = 1;
                ++changes;
              }
            }
          }
          // (additions spread over two or three bins are still cheaper singly)
          const uint32_t first_bin = (uint32_t)__builtin_amdgcn_readfirstlane((int)run_bin);
          by_ballot = __popcll((unsigned long long)__ballot(changes >= 3 && run_bin == first_bin)) >= 56;
          if (by_ballot) {
            if (run_cnt) atomicAdd(&hist[run_bin], run_cnt);
            run_cnt = 0;
          }
        } else {
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int t = (cb + u) * 64 + lane;
            bool todo = cb + u < pc1 && t < S && (kk[u] & known) == prefix;
            const uint32_t bin = (kk[u] >> shift) & (uint32_t)(bins - 1);
#pragma unroll
            for (int round = 0; round < 3; ++round) {
              const uint64_t left = __ballot(todo);
              if (left == 0) break;
              const uint32_t lead = (uint32_t)__shfl((int)bin, __ffsll((unsigned long long)left) - 1);
              const uint64_t same = __ballot(todo && bin == lead);
              if (todo && bin == lead) {
                if ((same & lanemask_lt()) == 0) atomicAdd(&hist[lead], (uint32_t)__popcll(same));
                todo = false;
              }
            }
            if (todo) atomicAdd(&hist[bin], 1u);
          }
        }
      }
      if (run_cnt) atomicAdd(&hist[run_bin], run_cnt);
    }
    __syncthreads();
    // thread i owns bins (bins-1 - per*i) downwards; `above` = keys with a larger digit
    const int per = bins / kSelThreads;  // 2, 2, 1
    uint32_t c[2] = {0u, 0u};
    int local = 0;
    for (int j = 0; j < per; ++j) {
      const int bin = bins - 1 - per * tid - j;
      c[j] = hist[bin];
      hist[bin] = 0;  // ready for the next pass
      local += (int)c[j];
    }
    uint32_t above = (uint32_t)block_excl_scan(local, wave_tot);
    for (int j = 0; j < per; ++j) {
      if (above < remaining && remaining <= above + c[j]) {
        sh_digit = (uint32_t)(bins - 1 - per * tid - j);
        sh_remaining = remaining - above;
        sh_count = c[j];
      }
      above += c[j];
    }
    __syncthreads();
    prefix |= sh_digit << shift;
    known |= (uint32_t)(bins - 1) << shift;
    remaining = sh_remaining;
  }
  const uint32_t T = prefix;          // key of the k-th largest element
  const uint32_t count_eq = sh_count; // elements equal to it; `remaining` of them are taken

  int c0, c1;
  wave_chunk_range(nw, kSelWaves, wave, c0, c1);
  int eq_before = 0;
  const bool ties = count_eq != remaining;  // uniform over the workgroup
  // (chunks are taken four at a time so that their key reads overlap)
  if (ties) {
    int mine = 0;
    for (int cb = c0; cb < c1; cb += 4) {
      uint32_t kk[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int t = (cb + u) * 64 + lane;
        kk[u] = (cb + u < c1 && t < S) ? key_at(t) : ~T;  // ~T never equals T
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) mine += kk[u] == T ? 1 : 0;
    }
    mine = wave_sum(mine);
    if (lane == 0) wave_tot[wave] = mine;
    __syncthreads();
    for (int w = 0; w < wave; ++w) eq_before += wave_tot[w];
  }
  for (int cb = c0; cb < c1; cb += 4) {
    uint32_t kk[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int t = (cb + u) * 64 + lane;
      kk[u] = (cb + u < c1 && t < S) ? key_at(t) : 0u;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int c = cb + u;
      if (c >= c1) break;  // uniform
      const int t = c * 64 + lane;
      const uint32_t key = kk[u];
      bool sel = t < S && key >= T;
      if (ties) {
        const bool eq = t < S && key == T;
        const uint64_t m = __ballot(eq);
        const int rank = eq_before + __popcll(m & lanemask_lt());
        if (eq) sel = rank < (int)remaining;
        eq_before += __popcll(m);
      }
      const uint64_t word = __ballot(sel);
      if (lane == 0) mask_out[c] = word;
    }
  }
}

// ------------------------------------------------------------- K1b (units) --
// Chunk- / page-level selection (Sec. 4.3.4, 4.3.5): the binary vector of a unit
// of `unit` tokens is the concatenation of its tokens' head vectors, bit
// j * Hs + r = head r of the unit's j-th token.  Rewritten as bitmaps over units,
// that is Hs * unit "virtual rows": row j * Hs + r holds, for unit u, bit
// u * unit + j of token row r.  After this de-interleave the grouping kernels
// run on units exactly as they do on tokens.
struct UnitRowsParams {
  const uint64_t* rowmask_tok;  // [B,Hs+1,nw_tok]; row Hs: important UNITS in its first nw_unit words
  uint64_t* rowmask_unit;       // [B,Hs*unit+1,nw_unit]
  int Hs, unit, n_units, nw_tok, nw_unit;
};

__global__ __launch_bounds__(256) void unit_rows_kernel(UnitRowsParams p) {
  const int b = blockIdx.y, lane = lane_id();
  const int Hv = p.Hs * p.unit;
  const uint64_t* __restrict__ src = p.rowmask_tok + (size_t)b * (p.Hs + 1) * p.nw_tok;
  uint64_t* __restrict__ dst = p.rowmask_unit + (size_t)b * (Hv + 1) * p.nw_unit;
  // one wave per output word
  const long long n_words = (long long)(Hv + 1) * p.nw_unit;
  const long long wave0 = (long long)blockIdx.x * 4 + threadIdx.x / KVC_WAVE;
  for (long long i = wave0; i < n_words; i += (long long)gridDim.x * 4) {
    const int row = (int)(i / p.nw_unit), c = (int)(i % p.nw_unit);
    uint64_t word;
    if (row == Hv) {
      word = src[(size_t)p.Hs * p.nw_tok + c];
    } else {
      const int j = row / p.Hs, r = row % p.Hs;
      const int u = c * 64 + lane;
      bool bit = false;
      if (u < p.n_units) {
        const long long t = (long long)u * p.unit + j;
        bit = (src[(size_t)r * p.nw_tok + (t >> 6)] >> (t & 63)) & 1ull;
      }
      word = __ballot(bit);
    }
    if (lane == 0) dst[i] = word;
  }
}

// ------------------------------------------------------------------ K2 ----
// The grouping of one sequence is spread over many small workgroups: the token
// range is dealt out in contiguous runs of 64-token chunks to "global waves"
// (workgroup x wave); K2a leaves, per token, its distance and its rank among
// the same-distance tokens of its own wave, plus a (distance, global wave)
// count table; K2b turns the table into start ranks and scatters.
constexpr int kGsThreads = 256;
constexpr int kGsWaves = kGsThreads / KVC_WAVE;
constexpr int kGsChunksPerWg = 16;  // 64-item chunks a workgroup takes (4 for long bit vectors, whose
                                    // per-item work is large and whose item counts are small)
constexpr uint32_t kNotGrouped = 0xFFFFFFFFu;
// Internal anchor mode: the mean anchor when no bit can reach a majority.  A bit is set in at
// most bit_topk items, so with 2 * bit_topk <= N (the usual case: the kept share of a row is
// well under half) the strict-majority anchor is all zeros and the per-row counts over the
// whole sequence need not be taken.
constexpr int kAnchorZero = 100;
constexpr int kDistBits = 12;  // distances range over 0..kMaxHs

struct GroupParams {
  const uint64_t* rowmask;      // [B,Hs+1,nw]
  uint64_t* bits;               // words of token 0 of sequence 0; sequences are bits_stride tokens apart
  size_t bits_stride;
  uint32_t* dist_rank;          // [B,S]: distance | rank-in-wave << kDistBits, or kNotGrouped
  int32_t* counts;              // [B,Hs+1,n_gw] tokens per (distance, global wave)
  int32_t* order;               // [B,S]: first N entries = grouped tokens by (d,t)
  uint64_t* repmask;            // [B,nw], zeroed by K2a
  const uint64_t* anchor_bits;  // [B,W] explicit anchor or null
  uint64_t anchor_seed;
  int Hs, S, nw, W, N, anchor_mode, dbits;
  int n_gw;                     // global waves per sequence = workgroups x kGsWaves
};

__device__ __forceinline__ uint64_t splitmix64_next(uint64_t& state) {
  state += 0x9E3779B97F4A7C15ull;
  uint64_t z = state;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// WMAX: 64-bit words a bit vector may have (2 covers up to 128 score rows, kMaxW the page-level
// vectors); loops over the words are unrolled so that the words stay in registers.
template <int WMAX, int CPW>
__global__ __launch_bounds__(kGsThreads) void group_rank_kernel(GroupParams p) {
  extern __shared__ uint64_t lds_words[];       // this workgroup's slice [Hs+1][CPW]
  __shared__ int run[kGsWaves][WMAX * 64 + 1];  // per wave: tokens seen so far per distance
  __shared__ int head_cnt[WMAX * 64];
  __shared__ uint64_t sh_anchor[WMAX];

  const int b = blockIdx.y, tid = threadIdx.x, lane = lane_id(), wave = tid / KVC_WAVE;
  const int S = p.S, Hs = p.Hs, nw = p.nw, W = p.W;
  const uint64_t* __restrict__ rm = p.rowmask + (size_t)b * (Hs + 1) * nw;
  const int wg_c0 = blockIdx.x * CPW;
  const int wg_nc = min(CPW, nw - wg_c0);

  // this workgroup's words of every row -> LDS (read many times below)
  for (int i = tid; i < (Hs + 1) * CPW; i += kGsThreads) {
    const int r = i / CPW, c = i % CPW;
    lds_words[i] = c < wg_nc ? rm[(size_t)r * nw + wg_c0 + c] : 0ull;
  }
  for (int c = tid; c < wg_nc; c += kGsThreads) p.repmask[(size_t)b * nw + wg_c0 + c] = 0ull;
  for (int i = tid; i < kGsWaves * (WMAX * 64 + 1); i += kGsThreads) (&run[0][0])[i] = 0;
  // ---- anchor (Alg. 2, first step); every workgroup derives the same one
  if (p.anchor_mode == KVCRUSH_ANCHOR_MEAN) {
    // bit r set in more than half of the grouped tokens?  counts over the whole sequence (these
    // loads share their latency with the staging loads above; head_cnt[r], r < Hs, is written here
    // and read only after the barrier)
    const uint64_t* __restrict__ imp = rm + (size_t)Hs * nw;
    for (int r = wave; r < Hs; r += kGsWaves) {
      int cnt = 0;
      for (int c = lane; c < nw; c += KVC_WAVE) cnt += __popcll(rm[(size_t)r * nw + c] & ~imp[c]);
      cnt = wave_sum(cnt);
      if (lane == 0) head_cnt[r] = cnt;
    }
  }
  __syncthreads();
  if (tid < W) {
    uint64_t a = 0;
    if (p.anchor_mode == KVCRUSH_ANCHOR_RANDOM) {
      uint64_t st = p.anchor_seed + (uint64_t)b;
      for (int w = 0; w <= tid; ++w) a = splitmix64_next(st);
    } else if (p.anchor_mode == KVCRUSH_ANCHOR_ALTERNATING) {
      a = 0xAAAAAAAAAAAAAAAAull;
    } else if (p.anchor_mode == KVCRUSH_ANCHOR_EXPLICIT) {
      a = p.anchor_bits[(size_t)b * W + tid];
    } else if (p.anchor_mode == KVCRUSH_ANCHOR_MEAN) {
      for (int r = tid * 64; r < min(Hs, tid * 64 + 64); ++r)
        if (2ll * head_cnt[r] > (long long)p.N) a |= 1ull << (r - tid * 64);
    }  // (kAnchorZero: stays zero)
    const int live = Hs - tid * 64;  // meaningful bits in this word
    if (live < 64) a &= (1ull << live) - 1ull;
    sh_anchor[tid] = a;
  }
  __syncthreads();
  uint64_t anchor[WMAX];
#pragma unroll
  for (int w = 0; w < WMAX; ++w) anchor[w] = w < W ? sh_anchor[w] : 0ull;

  // ---- this wave's chunks: bit words out, distance, stable rank inside the wave
  const int gw = blockIdx.x * kGsWaves + wave;
  constexpr int kPerWave = CPW / kGsWaves;
  const int c0 = min(nw, wg_c0 + wave * kPerWave), c1 = min(nw, c0 + kPerWave);
  for (int c = c0; c < c1; ++c) {
    const int lc = c - wg_c0;
    const int t = c * 64 + lane;
    uint64_t bw[WMAX];
    uint32_t d = 0;
#pragma unroll
    for (int w = 0; w < WMAX; ++w) {
      uint64_t acc = 0ull;
      const int nb = min(64, Hs - 64 * w);  // rows in this word (<= 0: none)
      for (int rr = 0; rr < nb; ++rr) {
        const uint64_t word = lds_words[(64 * w + rr) * CPW + lc];  // same address for the whole wave
        acc |= ((word >> lane) & 1ull) << rr;
      }
      bw[w] = acc;
      d += (uint32_t)__popcll(acc ^ anchor[w]);
    }
    const bool grouped = t < S && !((lds_words[Hs * CPW + lc] >> lane) & 1ull);
    if (t < S) {
#pragma unroll
      for (int w = 0; w < WMAX; ++w)
        if (w < W) p.bits[((size_t)b * p.bits_stride + t) * W + w] = bw[w];
    }
    const uint64_t peers = match_peers(d, p.dbits, grouped);
    uint32_t packed = kNotGrouped;
    if (grouped) {
      const int base = run[wave][d];
      packed = d | ((uint32_t)(base + __popcll(peers & lanemask_lt())) << kDistBits);
      if (lane == __ffsll((unsigned long long)peers) - 1) run[wave][d] = base + __popcll(peers);
    }
    if (t < S) p.dist_rank[(size_t)b * S + t] = packed;
  }
  // this wave's column of the count table
  for (int d = lane; d <= Hs; d += KVC_WAVE)
    p.counts[((size_t)b * (Hs + 1) + d) * p.n_gw + gw] = run[wave][d];
}

template <int CPW>
__global__ __launch_bounds__(kGsThreads) void group_scatter_kernel(GroupParams p) {
  extern __shared__ int lds_base[];  // [(Hs+1) * n_gw] start rank of every (distance, global wave)
  __shared__ int wave_tot[kGsWaves];

  const int b = blockIdx.y, tid = threadIdx.x, lane = lane_id(), wave = tid / KVC_WAVE;
  const int S = p.S, Hs = p.Hs, nw = p.nw;
  const int total = (Hs + 1) * p.n_gw;
  const int32_t* __restrict__ counts = p.counts + (size_t)b * total;

  // exclusive scan of the table in (distance, wave) order; every workgroup does the whole
  // (small) table itself rather than waiting for another launch
  const int per = (total + kGsThreads - 1) / kGsThreads;
  const int i0 = min(total, tid * per), i1 = min(total, i0 + per);
  int local = 0;
  for (int i = i0; i < i1; ++i) local += counts[i];
  {
    const int incl = wave_incl_scan(local);
    if (lane == KVC_WAVE - 1) wave_tot[wave] = incl;
    __syncthreads();
    int run = incl - local;
    for (int w = 0; w < wave; ++w) run += wave_tot[w];
    for (int i = i0; i < i1; ++i) {
      lds_base[i] = run;
      run += counts[i];
    }
  }
  __syncthreads();

  const int gw = blockIdx.x * kGsWaves + wave;
  constexpr int kPerWave = CPW / kGsWaves;
  const int c0 = min(nw, (int)blockIdx.x * CPW + wave * kPerWave), c1 = min(nw, c0 + kPerWave);
  int32_t* __restrict__ order = p.order + (size_t)b * S;
  for (int c = c0; c < c1; ++c) {
    const int t = c * 64 + lane;
    if (t < S) {
      const uint32_t packed = p.dist_rank[(size_t)b * S + t];
      if (packed != kNotGrouped)
        order[lds_base[(packed & ((1u << kDistBits) - 1u)) * p.n_gw + gw] + (int)(packed >> kDistBits)] = t;
    }
  }
}

// ------------------------------------------------------------------ K3 ----
struct MedoidParams {
  const uint64_t* bits;   // as in GroupParams
  size_t bits_stride;
  const int32_t* order;   // [B,S]
  uint64_t* repmask;      // [B,nw]
  int Hs, S, nw, W, N, Br;
};

constexpr int kMedoidThreads = 256;
constexpr int kMedoidWaves = kMedoidThreads / KVC_WAVE;

template <int WMAX>
__global__ __launch_bounds__(kMedoidThreads) void medoid_kernel(MedoidParams p) {
  const int b = blockIdx.y, lane = lane_id(), wave = threadIdx.x / KVC_WAVE;
  const int j = blockIdx.x * kMedoidWaves + wave;  // bucket of this wave
  if (j >= p.Br) return;
  const int W = p.W, Hs = p.Hs;
  const long long lo = (long long)j * p.N / p.Br, hi = (long long)(j + 1) * p.N / p.Br;
  const int n = (int)(hi - lo);
  const int32_t* order = p.order + (size_t)b * p.S + lo;
  const uint64_t* bits = p.bits + (size_t)b * p.bits_stride * W;

  // per-bit member counts: lane l keeps bits l, l + 64, ...
  int cnt[WMAX];
#pragma unroll
  for (int w = 0; w < WMAX; ++w) cnt[w] = 0;
  for (int m0 = 0; m0 < n; m0 += KVC_WAVE) {
    const int m = m0 + lane;
    const int t = m < n ? order[m] : 0;
#pragma unroll
    for (int w = 0; w < WMAX; ++w) {
      const uint64_t bw = (m < n && w < W) ? bits[(size_t)t * W + w] : 0ull;
      const int nb = min(64, Hs - 64 * w);
      for (int rr = 0; rr < nb; ++rr) {
        const int c = __popcll(__ballot((bw >> rr) & 1ull));
        if (lane == rr) cnt[w] += c;
      }
    }
  }
  // cost = summed Hamming distance to the members; keep (cost, token) minimum
  unsigned long long best = ~0ull;
  for (int m0 = 0; m0 < n; m0 += KVC_WAVE) {
    const int m = m0 + lane;
    const int t = m < n ? order[m] : 0;
    unsigned int cost = 0;
#pragma unroll
    for (int w = 0; w < WMAX; ++w) {
      const uint64_t bw = (m < n && w < W) ? bits[(size_t)t * W + w] : 0ull;
      const int nb = min(64, Hs - 64 * w);
      for (int rr = 0; rr < nb; ++rr) {
        const int c = __shfl(cnt[w], rr);
        cost += ((bw >> rr) & 1ull) ? (unsigned)(n - c) : (unsigned)c;
      }
    }
    if (m < n) {
      const unsigned long long key = ((unsigned long long)cost << 32) | (unsigned)t;
      best = key < best ? key : best;
    }
  }
#pragma unroll
  for (int off = KVC_WAVE / 2; off > 0; off >>= 1) {
    const unsigned long long o = __shfl_xor(best, off);
    best = o < best ? o : best;
  }
  if (lane == 0) {
    const int t = (int)(best & 0xFFFFFFFFull);
    atomicOr((unsigned long long*)&p.repmask[(size_t)b * p.nw + (t >> 6)], 1ull << (t & 63));
  }
}

// Long bit vectors (page level: few buckets, hundreds of bits): a workgroup per bucket, the
// four waves share the vector's words (wave w takes words w, w + 4, ...); counts stay inside a
// wave, the members' costs are added across the waves through LDS.
template <int WMAX>
__global__ __launch_bounds__(kMedoidThreads) void medoid_wide_kernel(MedoidParams p) {
  __shared__ unsigned int part[kMedoidWaves][KVC_WAVE];
  const int b = blockIdx.y, lane = lane_id(), wave = threadIdx.x / KVC_WAVE;
  const int j = blockIdx.x;  // bucket of this workgroup
  const int W = p.W, Hs = p.Hs;
  const long long lo = (long long)j * p.N / p.Br, hi = (long long)(j + 1) * p.N / p.Br;
  const int n = (int)(hi - lo);
  const int32_t* order = p.order + (size_t)b * p.S + lo;
  const uint64_t* bits = p.bits + (size_t)b * p.bits_stride * W;
  constexpr int kOwn = (WMAX + kMedoidWaves - 1) / kMedoidWaves;  // words a wave may own

  int cnt[kOwn];
#pragma unroll
  for (int o = 0; o < kOwn; ++o) cnt[o] = 0;
  for (int m0 = 0; m0 < n; m0 += KVC_WAVE) {
    const int m = m0 + lane;
    const int t = m < n ? order[m] : 0;
#pragma unroll
    for (int o = 0; o < kOwn; ++o) {
      const int w = wave + o * kMedoidWaves;
      const uint64_t bw = (m < n && w < W) ? bits[(size_t)t * W + w] : 0ull;
      const int nb = min(64, Hs - 64 * w);
      for (int rr = 0; rr < nb; ++rr) {
        const int c = __popcll(__ballot((bw >> rr) & 1ull));
        if (lane == rr) cnt[o] += c;
      }
    }
  }
  unsigned long long best = ~0ull;
  for (int m0 = 0; m0 < n; m0 += KVC_WAVE) {
    const int m = m0 + lane;
    const int t = m < n ? order[m] : 0;
    unsigned int cost = 0;
#pragma unroll
    for (int o = 0; o < kOwn; ++o) {
      const int w = wave + o * kMedoidWaves;
      const uint64_t bw = (m < n && w < W) ? bits[(size_t)t * W + w] : 0ull;
      const int nb = min(64, Hs - 64 * w);
      for (int rr = 0; rr < nb; ++rr) {
        const int c = __shfl(cnt[o], rr);
        cost += ((bw >> rr) & 1ull) ? (unsigned)(n - c) : (unsigned)c;
      }
    }
    part[wave][lane] = cost;
    __syncthreads();
    if (wave == 0 && m < n) {
      const unsigned int total = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
      const unsigned long long key = ((unsigned long long)total << 32) | (unsigned)t;
      best = key < best ? key : best;
    }
    __syncthreads();
  }
  if (wave == 0) {
#pragma unroll
    for (int off = KVC_WAVE / 2; off > 0; off >>= 1) {
      const unsigned long long o = __shfl_xor(best, off);
      best = o < best ? o : best;
    }
    if (lane == 0) {
      const int t = (int)(best & 0xFFFFFFFFull);
      atomicOr((unsigned long long*)&p.repmask[(size_t)b * p.nw + (t >> 6)], 1ull << (t & 63));
    }
  }
}

// ------------------------------------------------------------------ K4 ----
struct EmitParams {
  const uint64_t* impmask_base;  // rowmask + Hs*nw (row stride (Hs+1)*nw per sequence)
  const uint64_t* repmask;       // [B,nw]
  int32_t* idx;                  // [B,budget]
  uint8_t* kind;                 // nullable
  size_t imp_stride;
  int S, nw, budget;     // of the selectable (middle) tokens
  // protected ends: tokens [0, n_sink) and the last n_recent of the S_full tokens are kept
  // as they are; middle token u is token u + n_sink of the sequence
  int n_sink, n_recent, S_full, budget_full;
  uint64_t* bits_user;   // caller's bit words [B,S_full,W] or null: protected tokens get zero words
  int W;
  int unit;              // tokens per selected item: every kept item expands to `unit` indices
};

// The list of one sequence, written by one workgroup of NT threads: one bitmap word per
// thread, a prefix sum of the words' population counts, then the waves take the words in turn
// and the lanes whose bit is set write their item at its place, so that the stores of a wave
// go to consecutive entries.  Contains barriers: every thread of the workgroup calls it.
constexpr int kEmitTile = 1024;  // bitmap words handled per round (at most one per thread)
struct EmitScratch {             // LDS
  uint64_t kept[kEmitTile], rep[kEmitTile];
  int base[kEmitTile];
  int wave_tot[kSelWaves];
  int total;
};

template <int NT>
__device__ __forceinline__ void emit_sequence(const EmitParams& p, int b, EmitScratch& sh) {
  static_assert(NT <= kEmitTile, "one bitmap word per thread and round");
  constexpr int NW = NT / KVC_WAVE;
  const int tid = threadIdx.x, lane = lane_id(), wave = tid / KVC_WAVE;
  const uint64_t* imp = p.impmask_base + (size_t)b * p.imp_stride;
  const uint64_t* rep = p.repmask ? p.repmask + (size_t)b * p.nw : nullptr;  // null: no representatives
  int32_t* idx_out = p.idx + (size_t)b * p.budget_full;
  uint8_t* kind_out = p.kind ? p.kind + (size_t)b * p.budget_full : nullptr;
  for (int i = tid; i < p.n_sink + p.n_recent; i += NT) {
    const bool head = i < p.n_sink;
    const int o = head ? i : p.budget_full - p.n_recent + (i - p.n_sink);
    const int t = head ? i : p.S_full - p.n_recent + (i - p.n_sink);
    idx_out[o] = t;
    if (kind_out) kind_out[o] = 2;
    if (p.bits_user)
      for (int w = 0; w < p.W; ++w) p.bits_user[((size_t)b * p.S_full + t) * p.W + w] = 0ull;
  }
  idx_out += p.n_sink;
  if (kind_out) kind_out += p.n_sink;
  int carried = 0;  // items emitted by earlier rounds
  for (int w0 = 0; w0 < p.nw; w0 += NT) {
    const int c = w0 + tid;
    uint64_t rw = 0, kept = 0;
    if (c < p.nw) {
      rw = rep ? load_shared_word(rep + c) : 0ull;
      kept = load_shared_word(imp + c) | rw;
    }
    const int cnt = __popcll(kept);
    const int before = block_excl_scan(cnt, sh.wave_tot);
    sh.kept[tid] = kept;
    sh.rep[tid] = rw;
    sh.base[tid] = carried + before;
    if (tid == NT - 1) sh.total = before + cnt;
    __syncthreads();
    const int n_here = min(NT, p.nw - w0);
    constexpr int kAhead = 4;  // words whose LDS reads are in flight together (the loop is bound by their latency)
    for (int j0 = wave; j0 < n_here; j0 += NW * kAhead) {
      uint64_t kws[kAhead], reps[kAhead];
      int bases[kAhead];
#pragma unroll
      for (int a = 0; a < kAhead; ++a) {
        const int j = min(j0 + a * NW, NT - 1);
        kws[a] = sh.kept[j];
        reps[a] = sh.rep[j];
        bases[a] = sh.base[j];
      }
#pragma unroll
      for (int a = 0; a < kAhead; ++a) {
        const int j = j0 + a * NW;
        const uint64_t kw = j < n_here ? kws[a] : 0ull;
        if ((kw >> lane) & 1ull) {
          const int o = bases[a] + __popcll(kw & lanemask_lt());
          if (o < p.budget) {  // always true for consistent masks; keeps stores in bounds regardless
            const int item = (w0 + j) * 64 + lane;
            const uint8_t kd = (uint8_t)((reps[a] >> lane) & 1ull);
            if (p.unit == 1) {
              idx_out[o] = item + p.n_sink;
              if (kind_out) kind_out[o] = kd;
            } else {
              for (int e = 0; e < p.unit; ++e) {
                idx_out[(size_t)o * p.unit + e] = item * p.unit + e + p.n_sink;
                if (kind_out) kind_out[(size_t)o * p.unit + e] = kd;
              }
            }
          }
        }
      }
    }
    carried += sh.total;
    __syncthreads();
  }
}

__global__ __launch_bounds__(kSelThreads) void emit_kernel(EmitParams p) {
  __shared__ EmitScratch sh;
  emit_sequence<kSelThreads>(p, blockIdx.x, sh);
}

// =========================================== token-level selection in three launches ==
// The usual case (tokens, not units, as the selected items; at most 128 score rows; rows
// that fit the LDS tables below).  Every step that needs a view of a whole row or a whole
// sequence is a serial chain of short phases, so the stage is bound by how many such chains
// follow each other and by the fixed cost of a launch.  Three launches:
//
//   F1 slice_hist_kernel   the data-parallel part, spread over the chip: per (row, slice
//                          of 2048 tokens) the histogram of the keys' leading 11 bits; the
//                          importance row's workgroups first add up the score rows (in
//                          row order) and leave the sums in the workspace.
//   F2 row_select_kernel   one workgroup per row: adds the slices' histograms, finds the
//                          leading digit of the k-th key, settles the remaining 21 bits on
//                          the keys held in LDS, writes the row's bitmap.  The workgroup
//                          that finishes a sequence's LAST row goes on to group that
//                          sequence: bit words, anchor, distances and the stable counting
//                          sort by (distance, token), all in its LDS.
//   F3 medoid_emit_kernel  one wave per bucket picks the representative; the workgroup
//                          that finishes a sequence's LAST bucket writes the index list.
//
// "Last" is decided by an arrival counter in the workspace (an atomic add after a release
// fence; the counters are zeroed by F1, ahead of their first use in F2).  Nobody waits for
// anybody: a workgroup that is not the last simply ends.
constexpr int kSliceThreads = 256;
constexpr int kSliceTokens = 2048;  // tokens of one row handled by an F1 workgroup
constexpr int kFastMaxRows = 128;   // score rows (two 64-bit words per token)
constexpr int kFastMaxTokens = 32768;  // a row's keys live in its workgroup's registers: 1024 threads x 32

struct FastParams {
  const float* scores;   // first selectable token of row 0 of sequence 0; rows are `ld` floats apart
  float* imp;            // [B,S] token importances (F1 -> F2)
  uint16_t* phist;       // [B,Hs+1,nsl,2048] slice histograms (F1 -> F2)
  uint32_t* counters;    // [B,4]: rows finished, bucket workgroups finished
  uint64_t* rowmask;     // [B,Hs+1,nw]; row Hs = important tokens
  uint64_t* repmask;     // [B,nw]
  uint64_t* bits;        // words of token 0 of sequence 0; sequences are bits_stride tokens apart
  size_t bits_stride;
  int32_t* order;        // [B,S]: first N entries = grouped tokens by (distance, token)
  int Hs, S, nw, ld, kbit, n_important;
  int slice, nsl;        // tokens per slice, slices per row
  int row0, rows;        // rows handled: all Hs + 1, or the importance row alone
  int W, N, Br;
  int tail;              // 1: the row's workgroup writes the index list (plain top-n: no representatives)
  EmitParams emit;
};

// One LDS histogram addition per key, except that the lanes sharing the bin of the wave's
// first counted lane add once together: neighbouring scores are of similar size and equal keys
// share every digit, so this one round takes most of the same-address traffic away.
__device__ __forceinline__ void hist_add(uint32_t* hist, uint32_t bin, bool valid) {
  const uint64_t act = __ballot(valid);
  if (act == 0) return;  // uniform
  const int first = __ffsll((unsigned long long)act) - 1;
  const uint32_t lead = (uint32_t)__builtin_amdgcn_readlane((int)bin, first);
  const uint64_t same = __ballot(valid && bin == lead);
  if (valid) {
    if (bin == lead) {
      if (lane_id() == first) atomicAdd(&hist[lead], (uint32_t)__popcll(same));
    } else {
      atomicAdd(&hist[bin], 1u);
    }
  }
}

__global__ __launch_bounds__(kSliceThreads) void slice_hist_kernel(FastParams p) {
  __shared__ __align__(16) uint32_t hist[kRadixBins];
  const int s = blockIdx.x, row = p.row0 + blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  const int Hs = p.Hs;
  for (int i = tid; i < kRadixBins; i += kSliceThreads) hist[i] = 0;
  if (s == 0 && blockIdx.y == 0 && tid < 4) p.counters[(size_t)b * 4 + tid] = 0;
  __syncthreads();
  const float* __restrict__ sc = p.scores + (size_t)b * Hs * p.ld;
  const size_t ld = (size_t)p.ld;
  const int t0 = s * p.slice, t1 = min(p.S, t0 + p.slice);
  constexpr int kU = 8;  // tokens per thread in flight
  for (int base = t0 + tid; base < t1; base += kU * kSliceThreads) {
    float v[kU];
    if (row < Hs) {
#pragma unroll
      for (int u = 0; u < kU; ++u) {
        const int t = base + u * kSliceThreads;
        v[u] = t < t1 ? sc[(size_t)row * ld + t] : 0.0f;
      }
    } else {
      // token importance: fp32 sum of the score rows, taken in row order (eight rows' loads in
      // flight at a time; the additions stay in row order)
#pragma unroll
      for (int u = 0; u < kU; ++u) v[u] = 0.0f;
      int r = 0;
      for (; r + 8 <= Hs; r += 8) {
        float x[8][kU];
#pragma unroll
        for (int rr = 0; rr < 8; ++rr)
#pragma unroll
          for (int u = 0; u < kU; ++u) {
            const int t = base + u * kSliceThreads;
            x[rr][u] = t < t1 ? sc[(size_t)(r + rr) * ld + t] : 0.0f;
          }
#pragma unroll
        for (int rr = 0; rr < 8; ++rr)
#pragma unroll
          for (int u = 0; u < kU; ++u) v[u] = v[u] + x[rr][u];
      }
      for (; r < Hs; ++r) {
#pragma unroll
        for (int u = 0; u < kU; ++u) {
          const int t = base + u * kSliceThreads;
          const float x = t < t1 ? sc[(size_t)r * ld + t] : 0.0f;
          v[u] = v[u] + x;
        }
      }
#pragma unroll
      for (int u = 0; u < kU; ++u) {
        const int t = base + u * kSliceThreads;
        if (t < t1) p.imp[(size_t)b * p.S + t] = v[u];
      }
    }
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const int t = base + u * kSliceThreads;
      hist_add(hist, float_key(v[u]) >> 21, t < t1);
    }
  }
  __syncthreads();
  // eight bins per thread, as 16-bit counts (a slice has fewer than 65536 tokens)
  uint16_t* __restrict__ out = p.phist + (((size_t)b * (Hs + 1) + row) * p.nsl + s) * kRadixBins;
  const uint4 a = *(const uint4*)&hist[8 * tid], c = *(const uint4*)&hist[8 * tid + 4];
  uint4 w;
  w.x = a.x | (a.y << 16);
  w.y = a.z | (a.w << 16);
  w.z = c.x | (c.y << 16);
  w.w = c.z | (c.w << 16);
  *(uint4*)(out + 8 * tid) = w;
}

// F2: the k-th largest key of one row and the row's bitmap, by one workgroup.  The row's keys
// stay in registers (KPT per thread; thread (wave w, lane l) holds token l of the 64-token
// chunks w, w + 16, ...), the leading digit comes from the slices' histograms, and only the
// keys that share it (a few percent of the row) go through the two remaining digit passes:
// every wave keeps its own candidates in its own stretch of LDS (64 * KPT entries, enough
// for all of its keys).  One compute unit issues every instruction of the row's keys, about
// 0.1 us per instruction and key at 16 K keys, so the per-key loops are kept short.
template <int KPT>
__global__ __launch_bounds__(kSelThreads) void row_select_kernel(FastParams p) {
  extern __shared__ __align__(16) uint32_t cand[];  // [kSelWaves][64 * KPT] low 21 key bits of each wave's candidates
  __shared__ uint32_t hist[kRadixBins];
  __shared__ uint32_t sh_digit, sh_remaining, sh_count, sh_last;
  __shared__ int wave_tot[kSelWaves];
  __shared__ int chunk_eq[kSelWaves * KPT];  // ties only: keys equal to the threshold, per chunk

  const int row = p.row0 + blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x, lane = lane_id(), wave = tid / KVC_WAVE;
  const int Hs = p.Hs, S = p.S, nw = p.nw;
  const int k = row < Hs ? p.kbit : p.n_important;
  uint64_t* __restrict__ mask_out = p.rowmask + ((size_t)b * (Hs + 1) + row) * nw;
  const float* __restrict__ src =
      row < Hs ? p.scores + ((size_t)b * Hs + row) * p.ld : p.imp + (size_t)b * S;

  if (k == 0 || k == S) {  // nothing or everything: no search needed
    for (int c = tid; c < nw; c += kSelThreads) {
      uint64_t w = 0;
      if (k == S) {
        const int rem = S - c * 64;
        w = rem >= 64 ? ~0ull : ((1ull << rem) - 1ull);
      }
      store_shared_word(mask_out + c, w);
    }
  } else {
    // the row's keys (loads in flight while the histograms are added up); tokens past the end
    // read as the smallest key and are never selected (k <= S real keys rank above or beside them;
    // beside them only as key 0, where the lower token index wins)
    float v[KPT];
#pragma unroll
    for (int u = 0; u < KPT; ++u) {
      const int t = tid + u * kSelThreads;
      v[u] = t < S ? src[t] : 0.0f;
    }
    // leading digit: the slices' histograms added up.  Thread i owns bins 2047 - 2i and 2046 - 2i,
    // one 32-bit word of two 16-bit counts per slice.
    const uint32_t* __restrict__ ph =
        (const uint32_t*)(p.phist + ((size_t)b * (Hs + 1) + row) * p.nsl * kRadixBins);
    uint32_t c_hi = 0, c_lo = 0;
    for (int s = 0; s < p.nsl; ++s) {
      const uint32_t w = ph[(size_t)s * (kRadixBins / 2) + (kRadixBins / 2 - 1 - tid)];
      c_lo += w & 0xFFFFu;
      c_hi += w >> 16;
    }
    hist[2 * tid] = 0;
    hist[2 * tid + 1] = 0;
    uint32_t remaining = (uint32_t)k;
    {
      const uint32_t above = (uint32_t)block_excl_scan((int)(c_hi + c_lo), wave_tot);
      if (above < remaining && remaining <= above + c_hi) {
        sh_digit = (uint32_t)(kRadixBins - 1 - 2 * tid);
        sh_remaining = remaining - above;
        sh_count = c_hi;
      } else if (above + c_hi < remaining && remaining <= above + c_hi + c_lo) {
        sh_digit = (uint32_t)(kRadixBins - 2 - 2 * tid);
        sh_remaining = remaining - above - c_hi;
        sh_count = c_lo;
      }
    }
    __syncthreads();
    const uint32_t d1 = sh_digit;
    remaining = sh_remaining;
    // this wave's candidates (valid keys with the leading digit d1) -> its stretch of LDS
    uint32_t key[KPT];
    uint32_t* __restrict__ mine = cand + wave * (KVC_WAVE * KPT);
    int n_mine = 0;  // uniform over the wave
#pragma unroll
    for (int u = 0; u < KPT; ++u) {
      const int t = tid + u * kSelThreads;
      key[u] = t < S ? float_key(v[u]) : 0u;
      const bool is_cand = (key[u] >> 21) == d1 && t < S;
      const uint64_t m = __ballot(is_cand);
      if (is_cand) mine[n_mine + __popcll(m & lanemask_lt())] = key[u] & 0x1FFFFFu;
      n_mine += __popcll(m);
    }
    // the other 21 bits: two passes (11 and 10 bits) over the candidates that match the prefix so far
    // (a wave reads back only what it wrote itself, so no barrier is needed before the first pass)
    uint32_t low_prefix = 0, low_known = 0;
#pragma unroll
    for (int pass = 1; pass < 3; ++pass) {
      const int shift = pass == 1 ? 10 : 0;
      const int bins = pass == 1 ? 2048 : 1024;
      for (int i0 = 0; i0 < n_mine; i0 += KVC_WAVE) {
        const int i = i0 + lane;
        const uint32_t x = i < n_mine ? mine[i] : 0u;
        hist_add(hist, (x >> shift) & (uint32_t)(bins - 1), i < n_mine && (x & low_known) == low_prefix);
      }
      __syncthreads();
      // thread i owns bins (bins-1 - per*i) downwards; `above` = keys with a larger digit
      const int per = bins / kSelThreads;  // 2, 1
      uint32_t c[2] = {0u, 0u};
      int local = 0;
      for (int j = 0; j < per; ++j) {
        const int bin = bins - 1 - per * tid - j;
        c[j] = hist[bin];
        hist[bin] = 0;  // ready for the next pass
        local += (int)c[j];
      }
      uint32_t above = (uint32_t)block_excl_scan(local, wave_tot);
      for (int j = 0; j < per; ++j) {
        if (above < remaining && remaining <= above + c[j]) {
          sh_digit = (uint32_t)(bins - 1 - per * tid - j);
          sh_remaining = remaining - above;
          sh_count = c[j];
        }
        above += c[j];
      }
      __syncthreads();
      low_prefix |= sh_digit << shift;
      low_known |= (uint32_t)(bins - 1) << shift;
      remaining = sh_remaining;
    }
    const uint32_t T = (d1 << 21) | low_prefix;  // key of the k-th largest element
    const uint32_t count_eq = sh_count;          // elements equal to it; the first `remaining` of them are taken
    const bool ties = count_eq != remaining;     // uniform over the workgroup
    if (ties) {
      // keys equal to T ahead of each chunk, in token order (chunk c = wave + 16 u)
#pragma unroll
      for (int u = 0; u < KPT; ++u) {
        const int t = tid + u * kSelThreads;
        const uint64_t m = __ballot(t < S && key[u] == T);
        if (lane == 0) chunk_eq[wave + kSelWaves * u] = __popcll(m);
      }
      __syncthreads();
      const int own = tid < kSelWaves * KPT ? chunk_eq[tid] : 0;  // one chunk per thread covers them all
      const int before = block_excl_scan(own, wave_tot);
      if (tid < kSelWaves * KPT) chunk_eq[tid] = before;
      __syncthreads();
    }
    // the bitmap: lane u of the wave collects the word of the wave's u-th chunk
    uint64_t word_of_lane = 0;
#pragma unroll
    for (int u = 0; u < KPT; ++u) {
      const int t = tid + u * kSelThreads;
      bool sel = key[u] >= T && t < S;
      if (ties) {
        const bool eq = t < S && key[u] == T;
        const uint64_t m = __ballot(eq);
        if (eq) sel = (int)chunk_eq[wave + kSelWaves * u] + __popcll(m & lanemask_lt()) < (int)remaining;
      }
      const uint64_t word = __ballot(sel);
      if (lane == u) word_of_lane = word;
    }
    if (lane < KPT && wave + kSelWaves * lane < nw) store_shared_word(mask_out + wave + kSelWaves * lane, word_of_lane);
  }

  // ---- plain top-n: the only row of the sequence goes straight on to the index list
  if (p.tail == 0) return;
  if (!arrive_last(&p.counters[(size_t)b * 4 + 0], (uint32_t)p.rows, &sh_last)) return;
  emit_sequence<kSelThreads>(p.emit, b, *reinterpret_cast<EmitScratch*>(cand));  // (the candidates are no longer needed)
}

// F3: representatives (one wave per bucket, as medoid_kernel), then the index list by the
// workgroup that finishes the sequence's last bucket.
__global__ __launch_bounds__(kSelThreads) void medoid_emit_kernel(FastParams p) {
  __shared__ EmitScratch sh;
  __shared__ uint32_t sh_last;
  const int b = blockIdx.y, lane = lane_id(), wave = threadIdx.x / KVC_WAVE;
  const int j = blockIdx.x * kSelWaves + wave;  // bucket of this wave
  const int W = p.W, Hs = p.Hs;
  if (j < p.Br) {
    const long long lo = (long long)j * p.N / p.Br, hi = (long long)(j + 1) * p.N / p.Br;
    const int n = (int)(hi - lo);
    const int32_t* order = p.order + (size_t)b * p.S + lo;
    const uint64_t* bits = p.bits + (size_t)b * p.bits_stride * W;
    // per-bit member counts: lane l keeps bits l and l + 64
    int cnt[2] = {0, 0};
    for (int m0 = 0; m0 < n; m0 += KVC_WAVE) {
      const int m = m0 + lane;
      const int t = m < n ? min(max(order[m], 0), p.S - 1) : 0;
#pragma unroll
      for (int w = 0; w < 2; ++w) {
        const uint64_t bw = (m < n && w < W) ? bits[(size_t)t * W + w] : 0ull;
        const int nb = min(64, Hs - 64 * w);
        for (int rr = 0; rr < nb; ++rr) {
          const int c = __popcll(__ballot((bw >> rr) & 1ull));
          if (lane == rr) cnt[w] += c;
        }
      }
    }
    // cost = summed Hamming distance to the members; keep the (cost, token) minimum
    unsigned long long best = ~0ull;
    for (int m0 = 0; m0 < n; m0 += KVC_WAVE) {
      const int m = m0 + lane;
      const int t = m < n ? min(max(order[m], 0), p.S - 1) : 0;
      unsigned int cost = 0;
#pragma unroll
      for (int w = 0; w < 2; ++w) {
        const uint64_t bw = (m < n && w < W) ? bits[(size_t)t * W + w] : 0ull;
        const int nb = min(64, Hs - 64 * w);
        for (int rr = 0; rr < nb; ++rr) {
          const int c = __shfl(cnt[w], rr);
          cost += ((bw >> rr) & 1ull) ? (unsigned)(n - c) : (unsigned)c;
        }
      }
      if (m < n) {
        const unsigned long long key = ((unsigned long long)cost << 32) | (unsigned)t;
        best = key < best ? key : best;
      }
    }
#pragma unroll
    for (int off = KVC_WAVE / 2; off > 0; off >>= 1) {
      const unsigned long long o = __shfl_xor(best, off);
      best = o < best ? o : best;
    }
    if (lane == 0) {
      const int t = (int)(best & 0xFFFFFFFFull);
      atomicOr((unsigned long long*)&p.repmask[(size_t)b * p.nw + (t >> 6)], 1ull << (t & 63));
    }
  }
  if (!arrive_last(&p.counters[(size_t)b * 4 + 1], gridDim.x, &sh_last)) return;
  emit_sequence<kSelThreads>(p.emit, b, sh);
}

// ------------------------------------------------------------- host side ---
// What the kernels work on.  K1 ranks TOKENS (the middle ones, when ends are
// protected) per score row; the grouping, the representatives and the emitted
// list work on ITEMS: tokens, or units of `unit` tokens whose bit vectors have
// Hs * unit bits.
struct SelectPlan {
  int unit, S_tok, nw_tok;     // tokens between the protected ends, their 64-token words
  int n_items, nw, Hv, W;      // items, their 64-item words, bits per item, 64-bit words per item
  int budget_items, imp_items; // kept / important items
  int cpw, n_wg, n_gw;         // chunks per grouping workgroup, workgroups / global waves per sequence
  bool keys_in_lds;
  // three-launch path (tokens as items, few score rows, tables that fit LDS)
  bool fast;
  int slice, nsl;              // tokens per histogram slice, slices per row
  // workspace offsets
  size_t rowmask_tok, rowmask, repmask, bits, order, dist_rank, counts, keys, imp, phist, counters, total;
};

// The radix select keeps a row's keys in LDS when they fit beside the static
// arrays (160 KiB of LDS per workgroup on gfx950); longer rows go through the
// workspace instead.
constexpr int kLdsKeyCapacity = 36864;  // 144 KiB of keys

bool select_args_ok(const kvcrush_select_args* a) {
  if (!a) return false;
  if (a->B < 1 || a->Hs < 1 || a->S < 1) return false;
  if (a->budget < 0 || a->budget > a->S) return false;
  if (a->score_stride != 0 && a->score_stride < a->S) return false;
  if (a->n_sink < 0 || a->n_recent < 0 || (long long)a->n_sink + a->n_recent > a->budget) return false;
  const int prot = a->n_sink + a->n_recent;
  if (a->n_important < 0 || a->n_important > a->budget - prot) return false;
  if (a->bit_topk < 0 || a->bit_topk > a->S - prot) return false;
  if (a->anchor < KVCRUSH_ANCHOR_RANDOM || a->anchor > KVCRUSH_ANCHOR_EXPLICIT) return false;
  if (a->anchor == KVCRUSH_ANCHOR_EXPLICIT && !a->anchor_bits) return false;
  if (a->unit < 0) return false;
  const int unit = a->unit > 1 ? a->unit : 1;
  if ((a->S - prot) % unit != 0 || (a->budget - prot) % unit != 0 || a->n_important % unit != 0)
    return false;
  return true;
}

// Sizes supported by the kernels (beyond what the arguments' own consistency demands).
bool select_args_supported(const kvcrush_select_args* a) {
  const long long unit = a->unit > 1 ? a->unit : 1;
  if (a->B > 65535) return false;  // sequences are the second grid dimension
  return a->Hs * unit <= kMaxHs;
}

SelectPlan select_plan(const kvcrush_select_args* a, bool need_bits_ws) {
  SelectPlan P;
  P.unit = a->unit > 1 ? a->unit : 1;
  P.S_tok = a->S - a->n_sink - a->n_recent;
  P.nw_tok = (P.S_tok + 63) / 64;
  P.n_items = P.S_tok / P.unit;
  P.nw = (P.n_items + 63) / 64;
  P.Hv = a->Hs * P.unit;
  P.W = (P.Hv + 63) / 64;
  P.budget_items = (a->budget - a->n_sink - a->n_recent) / P.unit;
  P.imp_items = a->n_important / P.unit;
  P.keys_in_lds = P.S_tok <= kLdsKeyCapacity;
  // long vectors: a quarter of the chunks per workgroup, as long as the scatter's count table
  // ((bits + 1) x global waves) still fits LDS
  P.cpw = kGsChunksPerWg;
  if (P.W > 2 && (size_t)(P.Hv + 1) * ((P.nw + 3) / 4) * kGsWaves * 4 <= 96 * 1024) P.cpw = 4;
  // short vectors: as many workgroups as the count table allows (the stage is latency bound)
  if (P.W <= 2 && (size_t)(P.Hv + 1) * ((P.nw + 3) / 4) * kGsWaves * 4 <= 48 * 1024) P.cpw = 4;
  P.n_wg = (P.nw + P.cpw - 1) / P.cpw;
  P.n_gw = P.n_wg * kGsWaves;
  const size_t B = (size_t)a->B;
  size_t off = 0;
  P.rowmask_tok = off;
  off += kvc::align_up(B * (a->Hs + 1) * P.nw_tok * 8, 256);
  P.rowmask = P.rowmask_tok;  // token level: the same bitmaps
  if (P.unit > 1) {
    P.rowmask = off;
    off += kvc::align_up(B * (P.Hv + 1) * P.nw * 8, 256);
  }
  P.repmask = off;
  off += kvc::align_up(B * P.nw * 8, 256);
  P.order = off;
  off += kvc::align_up(B * P.n_items * 4, 256);
  P.dist_rank = off;
  off += kvc::align_up(B * P.n_items * 4, 256);
  P.counts = off;
  off += kvc::align_up(B * (P.Hv + 1) * P.n_gw * 4, 256);
  P.bits = off;
  if (need_bits_ws) off += kvc::align_up(B * P.n_items * P.W * 8, 256);
  P.keys = off;
  if (!P.keys_in_lds) off += kvc::align_up(B * (a->Hs + 1) * P.S_tok * 4, 256);
  // the short path: per-slice histograms, token importances, arrival counters
  P.slice = kSliceTokens;
  P.nsl = P.S_tok > 0 ? (P.S_tok + P.slice - 1) / P.slice : 0;
  P.fast = P.unit == 1 && a->Hs <= kFastMaxRows && P.S_tok > 0 && P.S_tok <= kFastMaxTokens;
  P.imp = off;
  if (P.fast) off += kvc::align_up(B * P.S_tok * 4, 256);
  P.phist = off;
  if (P.fast) off += kvc::align_up(B * (a->Hs + 1) * P.nsl * kRadixBins * 2, 256);
  P.counters = off;
  if (P.fast) off += kvc::align_up(B * 16, 256);
  P.total = off;
  return P;
}

// LDS tables of the grouping: (bits + 1) x chunk words of a workgroup, and the scatter's
// (bits + 1) x global waves counters (the limit stated in the header).
bool plan_fits_lds(const SelectPlan& P) {
  return (size_t)(P.Hv + 1) * P.cpw * 8 <= 136 * 1024 && (size_t)(P.Hv + 1) * P.n_gw * 4 <= 120 * 1024;
}

template <int WMAX, int CPW>
kvcrush_status launch_grouping(const GroupParams& g, const MedoidParams& m, const SelectPlan& P, int B,
                               int Br, bool with_medoid, hipStream_t stream) {
  const size_t dyn_a = (size_t)(P.Hv + 1) * CPW * 8;
  const size_t dyn_b = (size_t)(P.Hv + 1) * P.n_gw * 4;
  // (everything that can fail on the host comes before the first launch)
  if (dyn_a > 32 * 1024 && kvc::allow_large_lds<group_rank_kernel<WMAX, CPW>>(24 * 1024) != KVCRUSH_OK)
    return KVCRUSH_ERR_HIP;
  if (dyn_b > 32 * 1024 && kvc::allow_large_lds<group_scatter_kernel<CPW>>(1024) != KVCRUSH_OK)
    return KVCRUSH_ERR_HIP;
  kvcrush_status st = kvc::launch(group_rank_kernel<WMAX, CPW>, dim3(P.n_wg, B), dim3(kGsThreads), dyn_a, stream, g);
  if (st != KVCRUSH_OK || Br == 0) return st;  // the rank order only serves the representatives
  st = kvc::launch(group_scatter_kernel<CPW>, dim3(P.n_wg, B), dim3(kGsThreads), dyn_b, stream, g);
  if (st != KVCRUSH_OK || !with_medoid) return st;
  if (WMAX > 2 && Br <= 65535) return kvc::launch(medoid_wide_kernel<WMAX>, dim3(Br, B), dim3(kMedoidThreads), 0, stream, m);
  return kvc::launch(medoid_kernel<WMAX>, dim3((Br + kMedoidWaves - 1) / kMedoidWaves, B), dim3(kMedoidThreads), 0,
                     stream, m);
}

}  // namespace

extern "C" size_t kvcrush_select_workspace(const kvcrush_select_args* args) {
  if (!select_args_ok(args) || !select_args_supported(args)) return 0;
  // sized for the case where the caller does not ask for the bit words
  const SelectPlan P = select_plan(args, true);
  return plan_fits_lds(P) ? P.total : 0;
}

namespace {
kvcrush_status select_run(const kvcrush_select_args* args, const float* scores, int32_t* idx,
                          uint8_t* kind, uint64_t* bits, void* workspace, size_t workspace_bytes,
                          void* hip_stream);
}  // namespace

extern "C" kvcrush_status kvcrush_select(const kvcrush_select_args* args, const float* scores,
                                         int32_t* idx, uint8_t* kind, uint64_t* bits,
                                         void* workspace, size_t workspace_bytes,
                                         void* hip_stream) {
  return select_run(args, scores, idx, kind, bits, workspace, workspace_bytes, hip_stream);
}

// ---------------------------------------------- selection without a workspace --
// For callers that cannot allocate (code under HIP graph capture, tight serving
// loops): the same kernels on a scratch array that is part of the library's
// device image.  Host code may not use the array's name as an address; the
// device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[KVCRUSH_SELECT_STATIC_MAX_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex static_scratch_mutex;
void* static_scratch_ptr[kMaxDevices] = {};

// Device address of this device's copy of `scratch` (each GPU holds its own), or null.
void* static_scratch_for_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(static_scratch_mutex);
  if (!static_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    static_scratch_ptr[dev] = ptr;
  }
  return static_scratch_ptr[dev];
}
}  // namespace

extern "C" kvcrush_status kvcrush_select_static(const kvcrush_select_args* args, const float* scores,
                                                int32_t* idx, uint8_t* kind, uint64_t* bits,
                                                void* hip_stream) {
  if (!select_args_ok(args)) return KVCRUSH_ERR_INVALID_ARG;
  if (!select_args_supported(args)) return KVCRUSH_ERR_UNSUPPORTED;
  // (every buffer of the workspace, the arrival counters included, is written inside a call
  // before that call reads it, so the previous call's contents need no clearing)
  const SelectPlan P = select_plan(args, bits == nullptr);
  if (!plan_fits_lds(P)) return KVCRUSH_ERR_UNSUPPORTED;
  if (P.total > (size_t)KVCRUSH_SELECT_STATIC_MAX_BYTES) return KVCRUSH_ERR_WORKSPACE;
  void* ptr = static_scratch_for_current_device();
  if (!ptr) return KVCRUSH_ERR_HIP;
  return select_run(args, scores, idx, kind, bits, ptr, (size_t)KVCRUSH_SELECT_STATIC_MAX_BYTES, hip_stream);
}

namespace {
kvcrush_status select_run(const kvcrush_select_args* args, const float* scores, int32_t* idx,
                          uint8_t* kind, uint64_t* bits, void* workspace, size_t workspace_bytes,
                          void* hip_stream) {
  if (!select_args_ok(args)) return KVCRUSH_ERR_INVALID_ARG;
  if (!select_args_supported(args)) return KVCRUSH_ERR_UNSUPPORTED;
  if (!scores || (!idx && args->budget > 0)) return KVCRUSH_ERR_INVALID_ARG;
  if (!kvc::aligned16(scores) || !kvc::aligned16(workspace) || (bits && !kvc::aligned16(bits)))
    return KVCRUSH_ERR_INVALID_ARG;
  const SelectPlan P = select_plan(args, bits == nullptr);
  if (P.total > 0 && (!workspace || workspace_bytes < P.total)) return KVCRUSH_ERR_WORKSPACE;
  if (!plan_fits_lds(P)) return KVCRUSH_ERR_UNSUPPORTED;

  hipStream_t stream = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  const int B = args->B, Hs = args->Hs, S_full = args->S;
  const int Br = P.budget_items - P.imp_items, N = P.n_items - P.imp_items;
  const int kbit = args->bit_topk == 0 ? args->budget - args->n_sink - args->n_recent : args->bit_topk;
  uint64_t* rowmask_tok = (uint64_t*)(ws + P.rowmask_tok);
  uint64_t* rowmask = (uint64_t*)(ws + P.rowmask);
  uint64_t* repmask = (uint64_t*)(ws + P.repmask);
  int32_t* order = (int32_t*)(ws + P.order);
  // caller's bit words: [B,S,W] per token (protected tokens included), or [B,n_items,W] per unit
  const bool token_level = P.unit == 1;
  uint64_t* bits_buf = !bits ? (uint64_t*)(ws + P.bits) : (token_level ? bits + (size_t)args->n_sink * P.W : bits);
  const size_t bits_stride = (bits && token_level) ? (size_t)S_full : (size_t)P.n_items;

  // Plain top-n (no representative budget, token level, bit words not asked for): only the importance
  // row is ranked and the grouping kernels have nothing to do.
  const bool plain_topk = Br == 0 && token_level && bits == nullptr;

  EmitParams ep;
  ep.impmask_base = rowmask + (size_t)P.Hv * P.nw;
  ep.repmask = plain_topk ? nullptr : repmask;
  ep.idx = idx;
  ep.kind = kind;
  ep.imp_stride = (size_t)(P.Hv + 1) * P.nw;
  ep.S = P.n_items;
  ep.nw = P.nw;
  ep.budget = P.budget_items;
  ep.n_sink = args->n_sink;
  ep.n_recent = args->n_recent;
  ep.S_full = S_full;
  ep.budget_full = args->budget;
  ep.bits_user = token_level ? bits : nullptr;
  ep.W = P.W;
  ep.unit = P.unit;

  const bool fast = P.fast && args->budget > 0;
  FastParams f;
  if (fast) {
    f.scores = scores + args->n_sink;
    f.imp = (float*)(ws + P.imp);
    f.phist = (uint16_t*)(ws + P.phist);
    f.counters = (uint32_t*)(ws + P.counters);
    f.rowmask = rowmask;
    f.repmask = repmask;
    f.bits = bits_buf;
    f.bits_stride = bits_stride;
    f.order = order;
    f.Hs = Hs;
    f.S = P.S_tok;
    f.nw = P.nw_tok;
    f.ld = args->score_stride ? args->score_stride : S_full;
    f.kbit = kbit;
    f.n_important = P.imp_items;
    f.slice = P.slice;
    f.nsl = P.nsl;
    f.row0 = plain_topk ? Hs : 0;
    f.rows = plain_topk ? 1 : Hs + 1;
    f.W = P.W;
    f.N = N;
    f.Br = Br;
    f.tail = plain_topk ? 1 : 0;
    f.emit = ep;
  }
  // large tables in LDS have to be allowed per kernel before the first launch of the call
  const bool kpt16 = P.S_tok <= 16 * kSelThreads;
  const size_t row_lds = (size_t)kSelThreads * (kpt16 ? 16 : 32) * 4;  // every key may be a candidate
  if (fast && (kpt16 ? kvc::allow_large_lds<row_select_kernel<16>>(16 * 1024)
                     : kvc::allow_large_lds<row_select_kernel<32>>(16 * 1024)) != KVCRUSH_OK)
    return KVCRUSH_ERR_HIP;
  if (!fast && P.n_items > 0 && P.keys_in_lds && (size_t)P.S_tok * 4 > 48 * 1024 &&
      kvc::allow_large_lds<topk_mask_kernel<true>>(12 * 1024) != KVCRUSH_OK)
    return KVCRUSH_ERR_HIP;

  // ---- per-row top-k -> row bitmaps
  if (fast) {
    kvcrush_status st = kvc::launch(slice_hist_kernel, dim3(P.nsl, f.rows, B), dim3(kSliceThreads), 0, stream, f);
    if (st != KVCRUSH_OK) return st;
    st = kpt16 ? kvc::launch(row_select_kernel<16>, dim3(f.rows, B), dim3(kSelThreads), row_lds, stream, f)
               : kvc::launch(row_select_kernel<32>, dim3(f.rows, B), dim3(kSelThreads), row_lds, stream, f);
    if (st != KVCRUSH_OK || plain_topk) return st;  // (plain top-n: the row's workgroup wrote the list)
  } else if (P.n_items > 0) {
    TopkParams p;
    p.scores = scores + args->n_sink;
    p.ld = args->score_stride ? args->score_stride : S_full;
    p.unit = P.unit;
    p.rowmask = rowmask_tok;
    p.keys_ws = P.keys_in_lds ? nullptr : (uint32_t*)(ws + P.keys);
    p.Hs = Hs;
    p.S = P.S_tok;
    p.nw = P.nw_tok;
    p.kbit = kbit;
    p.n_important = P.imp_items;
    p.importance_only = plain_topk ? 1 : 0;
    const kvcrush_status st =
        P.keys_in_lds ? kvc::launch(topk_mask_kernel<true>, dim3(Hs + 1, B), dim3(kSelThreads), (size_t)P.S_tok * 4, stream, p)
                      : kvc::launch(topk_mask_kernel<false>, dim3(Hs + 1, B), dim3(kSelThreads), 0, stream, p);
    if (st != KVCRUSH_OK) return st;
  }
  if (P.n_items > 0 && !token_level) {
    UnitRowsParams p;
    p.rowmask_tok = rowmask_tok;
    p.rowmask_unit = rowmask;
    p.Hs = Hs;
    p.unit = P.unit;
    p.n_units = P.n_items;
    p.nw_tok = P.nw_tok;
    p.nw_unit = P.nw;
    const long long words = (long long)(P.Hv + 1) * P.nw;
    const int gx = (int)std::min<long long>((words + 3) / 4, 2048);
    const kvcrush_status st = kvc::launch(unit_rows_kernel, dim3(gx, B), dim3(256), 0, stream, p);
    if (st != KVCRUSH_OK) return st;
  }
  // ---- bit words, distances, stable order by (distance, item); representatives
  if (P.n_items > 0 && !plain_topk) {
    GroupParams g;
    g.rowmask = rowmask;
    g.bits = bits_buf;
    g.bits_stride = bits_stride;
    g.dist_rank = (uint32_t*)(ws + P.dist_rank);
    g.counts = (int32_t*)(ws + P.counts);
    g.order = order;
    g.repmask = repmask;
    g.anchor_bits = args->anchor_bits;
    g.anchor_seed = args->anchor_seed;
    g.Hs = P.Hv;
    g.S = P.n_items;
    g.nw = P.nw;
    g.W = P.W;
    g.N = N;
    g.anchor_mode = args->anchor;
    // (token level only: a unit's bit is set in at most bit_topk units as well, but N counts units there)
    if (args->anchor == KVCRUSH_ANCHOR_MEAN && token_level && 2ll * kbit <= (long long)N) g.anchor_mode = kAnchorZero;
    int dbits = 0;
    while ((1 << dbits) <= P.Hv) ++dbits;  // distances range over 0..Hv
    g.dbits = dbits;
    g.n_gw = P.n_gw;
    MedoidParams m;
    m.bits = bits_buf;
    m.bits_stride = bits_stride;
    m.order = order;
    m.repmask = repmask;
    m.Hs = P.Hv;
    m.S = P.n_items;
    m.nw = P.nw;
    m.W = P.W;
    m.N = N;
    m.Br = Br;
    kvcrush_status st;
    if (P.W <= 2)
      st = P.cpw == 4 ? launch_grouping<2, 4>(g, m, P, B, Br, !fast, stream)
                      : launch_grouping<2, kGsChunksPerWg>(g, m, P, B, Br, !fast, stream);
    else if (P.W <= 4)
      st = P.cpw == 4 ? launch_grouping<4, 4>(g, m, P, B, Br, true, stream)
                      : launch_grouping<4, kGsChunksPerWg>(g, m, P, B, Br, true, stream);
    else
      st = P.cpw == 4 ? launch_grouping<kMaxW, 4>(g, m, P, B, Br, true, stream)
                      : launch_grouping<kMaxW, kGsChunksPerWg>(g, m, P, B, Br, true, stream);
    if (st != KVCRUSH_OK) return st;
  }
  // ---- the ascending index list
  if (fast)  // representatives and the list in one launch
    return kvc::launch(medoid_emit_kernel, dim3(std::max(1, (Br + kSelWaves - 1) / kSelWaves), B),
                       dim3(kSelThreads), 0, stream, f);
  if (args->budget > 0) return kvc::launch(emit_kernel, dim3(B), dim3(kSelThreads), 0, stream, ep);
  return KVCRUSH_OK;
}
}  // namespace
