// Stages 2-4 of the KVCrush step on gfx950: importance top-k, head-behaviour
// bit vectors (Alg. 1, Sec. 3.1), Hamming grouping and one representative per
// bucket (Alg. 2, Sec. 3.2), merged ascending index list.
//
// All integer / compare work on at most a few MiB, so the stage is bound by
// latency, not bandwidth: four short launches on one stream, no host round
// trip, no floating-point atomics (every tie is broken by token index, so the
// result is a pure function of the score tensor).
//
//   K1 topk_mask_kernel   one workgroup per (sequence, score row) plus one for
//                         the importance row: exact k-th largest by an 8-bit
//                         MSB-first radix select over order-preserving integer
//                         keys held in LDS, then a 64-tokens-per-word bitmap of
//                         the selected set (ties: lowest index first).
//   K2 group_sort_kernel  one workgroup per sequence: packs the row bitmaps
//                         into per-token words, builds the anchor, Hamming
//                         distance by xor+popcount, and a stable counting sort
//                         of the non-important tokens by distance (wave ballots
//                         give each token its rank among equal distances).
//   K3 medoid_kernel      one wavefront per bucket: per-head counts by ballot,
//                         integer cost, wave arg-min with token tie-break.
//   K4 emit_kernel        ordered compaction of (important | representative)
//                         bitmaps into the ascending index list.
#include "common.h"

namespace {

using kvc::lane_id;
using kvc::lanemask_lt;

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / KVC_WAVE;
constexpr int kMaxHs = 128;
constexpr int kMaxW = kMaxHs / 64;

// Order-preserving map from fp32 to uint32 (larger float -> larger key);
// -0.0 is folded onto +0.0 so that the two compare equal, as they do as floats.
__device__ __forceinline__ uint32_t float_key(float x) {
  uint32_t u = __float_as_uint(x);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int wave_incl_scan(int v) {
  const int lane = lane_id();
#pragma unroll
  for (int off = 1; off < KVC_WAVE; off <<= 1) {
    const int o = __shfl_up(v, off);
    if (lane >= off) v += o;
  }
  return v;
}

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int off = KVC_WAVE / 2; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
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

// ------------------------------------------------------------------ K1 ----
struct TopkParams {
  const float* scores;  // [B,Hs,S]
  uint64_t* rowmask;    // [B,Hs+1,nw]; row Hs = important tokens
  uint32_t* keys_ws;    // [B,Hs+1,S] when the row does not fit LDS, else null
  int Hs, S, nw, kbit, n_important;
};

__global__ __launch_bounds__(kSelThreads) void topk_mask_kernel(TopkParams p) {
  extern __shared__ uint32_t lds_keys[];
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sh_digit, sh_remaining, sh_count;
  __shared__ int wave_eq[kSelWaves];

  const int row = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x, lane = lane_id(), wave = tid / KVC_WAVE;
  const int S = p.S, Hs = p.Hs, nw = p.nw;
  const int k = row < Hs ? p.kbit : p.n_important;
  uint64_t* mask_out = p.rowmask + ((size_t)b * (Hs + 1) + row) * nw;

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

  uint32_t* keys = p.keys_ws ? p.keys_ws + ((size_t)b * (Hs + 1) + row) * S : lds_keys;
  const float* sc = p.scores + (size_t)b * Hs * S;
  if (row < Hs) {
    for (int t = tid; t < S; t += kSelThreads) keys[t] = float_key(sc[(size_t)row * S + t]);
  } else {
    // token importance: fp32 sum of the score rows, taken in row order
    for (int t = tid; t < S; t += kSelThreads) {
      float acc = 0.0f;
      for (int r = 0; r < Hs; ++r) acc = acc + sc[(size_t)r * S + t];
      keys[t] = float_key(acc);
    }
  }
  __syncthreads();

  // MSB-first radix select of the k-th largest key, 8 bits a pass.
  uint32_t prefix = 0, known = 0, remaining = (uint32_t)k;
  const int s_round = nw * 64;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int base = wave * 64; base < s_round; base += kSelThreads) {
      const int t = base + lane;
      const uint32_t key = t < S ? keys[t] : 0u;
      bool valid = t < S && (key & known) == prefix;
      const uint32_t digit = (key >> shift) & 255u;
      // Score exponents cluster, so most lanes of a wave share one or two
      // digits: count those by ballot, the rest by plain LDS atomics.
      uint64_t todo = __ballot(valid);
      for (int it = 0; it < 2 && todo; ++it) {
        const int leader = __ffsll((unsigned long long)todo) - 1;
        const uint32_t dl = __shfl(digit, leader);
        const uint64_t m = __ballot(valid && digit == dl);
        if (lane == leader) atomicAdd(&hist[dl], (uint32_t)__popcll(m));
        todo &= ~m;
        valid = valid && digit != dl;
      }
      if (valid) atomicAdd(&hist[digit], 1u);
    }
    __syncthreads();
    if (wave == 0) {
      // lane l owns bins 255-4l .. 252-4l; `above` = keys with a larger digit
      uint32_t c[4];
      int local = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        c[j] = hist[255 - 4 * lane - j];
        local += (int)c[j];
      }
      uint32_t above = (uint32_t)(wave_incl_scan(local) - local);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (above < remaining && remaining <= above + c[j]) {
          sh_digit = 255 - 4 * lane - j;
          sh_remaining = remaining - above;
          sh_count = c[j];
        }
        above += c[j];
      }
    }
    __syncthreads();
    prefix |= sh_digit << shift;
    known |= 255u << shift;
    remaining = sh_remaining;
  }
  const uint32_t T = prefix;          // key of the k-th largest element
  const uint32_t count_eq = sh_count; // elements equal to it; `remaining` of them are taken

  int c0, c1;
  wave_chunk_range(nw, kSelWaves, wave, c0, c1);
  int eq_before = 0;
  const bool ties = count_eq != remaining;  // uniform over the workgroup
  if (ties) {
    int mine = 0;
    for (int c = c0; c < c1; ++c) {
      const int t = c * 64 + lane;
      mine += (t < S && keys[t] == T) ? 1 : 0;
    }
    mine = wave_sum(mine);
    if (lane == 0) wave_eq[wave] = mine;
    __syncthreads();
    for (int w = 0; w < wave; ++w) eq_before += wave_eq[w];
  }
  for (int c = c0; c < c1; ++c) {
    const int t = c * 64 + lane;
    const uint32_t key = t < S ? keys[t] : 0u;
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

// ------------------------------------------------------------------ K2 ----
struct GroupParams {
  const uint64_t* rowmask;      // [B,Hs+1,nw]
  uint64_t* bits;               // [B,S,W]
  int32_t* order;               // [B,S]: first N entries = grouped tokens by (d,t)
  uint64_t* repmask;            // [B,nw], zeroed here
  const uint64_t* anchor_bits;  // [B,W] explicit anchor or null
  uint64_t anchor_seed;
  int Hs, S, nw, W, N, anchor_mode, dbits;
};

__device__ __forceinline__ uint64_t splitmix64_next(uint64_t& state) {
  state += 0x9E3779B97F4A7C15ull;
  uint64_t z = state;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

__global__ __launch_bounds__(kSelThreads) void group_sort_kernel(GroupParams p) {
  __shared__ int wcount[(kMaxHs + 1) * kSelWaves];  // [distance][wave]
  __shared__ int head_cnt[kMaxHs];
  __shared__ uint64_t sh_anchor[kMaxW];

  const int b = blockIdx.x, tid = threadIdx.x, lane = lane_id(), wave = tid / KVC_WAVE;
  const int S = p.S, Hs = p.Hs, nw = p.nw, W = p.W;
  const uint64_t* rm = p.rowmask + (size_t)b * (Hs + 1) * nw;
  const uint64_t* impmask = rm + (size_t)Hs * nw;

  for (int c = tid; c < nw; c += kSelThreads) p.repmask[(size_t)b * nw + c] = 0ull;
  for (int i = tid; i < (Hs + 1) * kSelWaves; i += kSelThreads) wcount[i] = 0;

  // ---- anchor (Alg. 2, first step)
  if (p.anchor_mode == KVCRUSH_ANCHOR_MEAN) {
    // bit r is set in more than half of the grouped tokens?
    for (int r = wave; r < Hs; r += kSelWaves) {
      int cnt = 0;
      for (int c = lane; c < nw; c += KVC_WAVE) cnt += __popcll(rm[(size_t)r * nw + c] & ~impmask[c]);
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
    } else {
      for (int r = tid * 64; r < min(Hs, tid * 64 + 64); ++r)
        if (2ll * head_cnt[r] > (long long)p.N) a |= 1ull << (r - tid * 64);
    }
    const int live = Hs - tid * 64;  // meaningful bits in this word
    if (live < 64) a &= (1ull << live) - 1ull;
    sh_anchor[tid] = a;
  }
  __syncthreads();
  uint64_t anchor[kMaxW];
#pragma unroll
  for (int w = 0; w < kMaxW; ++w) anchor[w] = w < W ? sh_anchor[w] : 0ull;

  // ---- pass 1: per-token bit words, distance histogram per wave
  int c0, c1;
  wave_chunk_range(nw, kSelWaves, wave, c0, c1);
  for (int c = c0; c < c1; ++c) {
    const int t = c * 64 + lane;
    uint64_t bw[kMaxW] = {0ull, 0ull};
    for (int r = 0; r < Hs; ++r) {
      const uint64_t word = rm[(size_t)r * nw + c];  // same address for the whole wave
      bw[r >> 6] |= ((word >> lane) & 1ull) << (r & 63);
    }
    const bool grouped = t < S && !((impmask[c] >> lane) & 1ull);
    if (t < S) {
      for (int w = 0; w < W; ++w) p.bits[((size_t)b * S + t) * W + w] = bw[w];
    }
    const uint32_t d = (uint32_t)(__popcll(bw[0] ^ anchor[0]) + __popcll(bw[1] ^ anchor[1]));
    const uint64_t peers = match_peers(d, p.dbits, grouped);
    if (grouped && lane == __ffsll((unsigned long long)peers) - 1)
      wcount[d * kSelWaves + wave] += __popcll(peers);
  }
  __syncthreads();

  // ---- exclusive scan over (distance, wave): start rank of each wave's run
  if (wave == 0) {
    const int total = (Hs + 1) * kSelWaves;
    const int per = (total + KVC_WAVE - 1) / KVC_WAVE;
    const int i0 = min(total, lane * per), i1 = min(total, i0 + per);
    int local = 0;
    for (int i = i0; i < i1; ++i) local += wcount[i];
    int run = wave_incl_scan(local) - local;
    for (int i = i0; i < i1; ++i) {
      const int v = wcount[i];
      wcount[i] = run;
      run += v;
    }
  }
  __syncthreads();

  // ---- pass 2: stable scatter into rank order
  int32_t* order = p.order + (size_t)b * S;
  for (int c = c0; c < c1; ++c) {
    const int t = c * 64 + lane;
    const bool grouped = t < S && !((impmask[c] >> lane) & 1ull);
    uint32_t d = 0;
    if (t < S) {
      for (int w = 0; w < W; ++w) d += __popcll(p.bits[((size_t)b * S + t) * W + w] ^ anchor[w]);
    }
    const uint64_t peers = match_peers(d, p.dbits, grouped);
    if (grouped) {
      const int slot = d * kSelWaves + wave;
      const int base = wcount[slot];
      order[base + __popcll(peers & lanemask_lt())] = t;
      if (lane == __ffsll((unsigned long long)peers) - 1) wcount[slot] = base + __popcll(peers);
    }
  }
}

// ------------------------------------------------------------------ K3 ----
struct MedoidParams {
  const uint64_t* bits;   // [B,S,W]
  const int32_t* order;   // [B,S]
  uint64_t* repmask;      // [B,nw]
  int Hs, S, nw, W, N, Br;
};

constexpr int kMedoidThreads = 256;
constexpr int kMedoidWaves = kMedoidThreads / KVC_WAVE;

__global__ __launch_bounds__(kMedoidThreads) void medoid_kernel(MedoidParams p) {
  const int b = blockIdx.y, lane = lane_id(), wave = threadIdx.x / KVC_WAVE;
  const int j = blockIdx.x * kMedoidWaves + wave;  // bucket of this wave
  if (j >= p.Br) return;
  const int W = p.W, Hs = p.Hs;
  const long long lo = (long long)j * p.N / p.Br, hi = (long long)(j + 1) * p.N / p.Br;
  const int n = (int)(hi - lo);
  const int32_t* order = p.order + (size_t)b * p.S + lo;
  const uint64_t* bits = p.bits + (size_t)b * p.S * W;

  // per-head member counts: lane l keeps heads l and l+64
  int cnt[kMaxW] = {0, 0};
  for (int m0 = 0; m0 < n; m0 += KVC_WAVE) {
    const int m = m0 + lane;
    uint64_t bw[kMaxW] = {0ull, 0ull};
    if (m < n) {
      const int t = order[m];
      for (int w = 0; w < W; ++w) bw[w] = bits[(size_t)t * W + w];
    }
    for (int r = 0; r < Hs; ++r) {
      const int c = __popcll(__ballot((bw[r >> 6] >> (r & 63)) & 1ull));
      if (lane == (r & 63)) cnt[r >> 6] += c;
    }
  }
  // cost = summed Hamming distance to the members; keep (cost, token) minimum
  unsigned long long best = ~0ull;
  for (int m0 = 0; m0 < n; m0 += KVC_WAVE) {
    const int m = m0 + lane;
    uint64_t bw[kMaxW] = {0ull, 0ull};
    int t = 0;
    if (m < n) {
      t = order[m];
      for (int w = 0; w < W; ++w) bw[w] = bits[(size_t)t * W + w];
    }
    unsigned int cost = 0;
    for (int r = 0; r < Hs; ++r) {
      const int c = __shfl(cnt[r >> 6], r & 63);
      cost += ((bw[r >> 6] >> (r & 63)) & 1ull) ? (unsigned)(n - c) : (unsigned)c;
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

// ------------------------------------------------------------------ K4 ----
struct EmitParams {
  const uint64_t* impmask_base;  // rowmask + Hs*nw (row stride (Hs+1)*nw per sequence)
  const uint64_t* repmask;       // [B,nw]
  int32_t* idx;                  // [B,budget]
  uint8_t* kind;                 // nullable
  size_t imp_stride;
  int S, nw, budget;
};

__global__ __launch_bounds__(kSelThreads) void emit_kernel(EmitParams p) {
  __shared__ int wave_tot[kSelWaves];
  const int b = blockIdx.x, lane = lane_id(), wave = threadIdx.x / KVC_WAVE;
  const uint64_t* imp = p.impmask_base + (size_t)b * p.imp_stride;
  const uint64_t* rep = p.repmask + (size_t)b * p.nw;
  int c0, c1;
  wave_chunk_range(p.nw, kSelWaves, wave, c0, c1);
  int mine = 0;
  for (int c = c0 + lane; c < c1; c += KVC_WAVE) mine += __popcll(imp[c] | rep[c]);
  mine = wave_sum(mine);
  if (lane == 0) wave_tot[wave] = mine;
  __syncthreads();
  int base = 0;
  for (int w = 0; w < wave; ++w) base += wave_tot[w];
  for (int c = c0; c < c1; ++c) {
    const uint64_t rw = rep[c], kept = imp[c] | rw;
    if ((kept >> lane) & 1ull) {
      const int o = base + __popcll(kept & lanemask_lt());
      if (o < p.budget) {  // always true for consistent masks; keeps stores in bounds regardless
        p.idx[(size_t)b * p.budget + o] = c * 64 + lane;
        if (p.kind) p.kind[(size_t)b * p.budget + o] = (uint8_t)((rw >> lane) & 1ull);
      }
    }
    base += __popcll(kept);
  }
}

// ------------------------------------------------------------- host side ---
struct SelectLayout {
  size_t rowmask, repmask, bits, order, keys, total;
  int nw, W;
  bool keys_in_lds;
};

// The radix select keeps a row's keys in LDS when they fit beside the static
// arrays (160 KiB of LDS per workgroup on gfx950); longer rows go through the
// workspace instead.
constexpr int kLdsKeyCapacity = 36864;  // 144 KiB of keys

SelectLayout select_layout(const kvcrush_select_args* a, bool need_bits_ws) {
  SelectLayout L;
  L.nw = (a->S + 63) / 64;
  L.W = (a->Hs + 63) / 64;
  L.keys_in_lds = a->S <= kLdsKeyCapacity;
  size_t off = 0;
  L.rowmask = off;
  off += kvc::align_up((size_t)a->B * (a->Hs + 1) * L.nw * 8, 256);
  L.repmask = off;
  off += kvc::align_up((size_t)a->B * L.nw * 8, 256);
  L.order = off;
  off += kvc::align_up((size_t)a->B * a->S * 4, 256);
  L.bits = off;
  if (need_bits_ws) off += kvc::align_up((size_t)a->B * a->S * L.W * 8, 256);
  L.keys = off;
  if (!L.keys_in_lds) off += kvc::align_up((size_t)a->B * (a->Hs + 1) * a->S * 4, 256);
  L.total = off;
  return L;
}

bool select_args_ok(const kvcrush_select_args* a) {
  if (!a) return false;
  if (a->B < 1 || a->Hs < 1 || a->S < 1) return false;
  if (a->budget < 0 || a->budget > a->S) return false;
  if (a->n_important < 0 || a->n_important > a->budget) return false;
  if (a->bit_topk < 0 || a->bit_topk > a->S) return false;
  if (a->anchor < KVCRUSH_ANCHOR_RANDOM || a->anchor > KVCRUSH_ANCHOR_EXPLICIT) return false;
  if (a->anchor == KVCRUSH_ANCHOR_EXPLICIT && !a->anchor_bits) return false;
  return true;
}

}  // namespace

extern "C" size_t kvcrush_select_workspace(const kvcrush_select_args* args) {
  if (!select_args_ok(args) || args->Hs > kMaxHs) return 0;
  // sized for the case where the caller does not ask for the bit words
  return select_layout(args, true).total;
}

extern "C" kvcrush_status kvcrush_select(const kvcrush_select_args* args, const float* scores,
                                         int32_t* idx, uint8_t* kind, uint64_t* bits,
                                         void* workspace, size_t workspace_bytes,
                                         void* hip_stream) {
  if (!select_args_ok(args)) return KVCRUSH_ERR_INVALID_ARG;
  if (args->Hs > kMaxHs) return KVCRUSH_ERR_UNSUPPORTED;
  if (!scores || (!idx && args->budget > 0)) return KVCRUSH_ERR_INVALID_ARG;
  if (!kvc::aligned16(scores) || !kvc::aligned16(workspace) || (bits && !kvc::aligned16(bits)))
    return KVCRUSH_ERR_INVALID_ARG;
  const SelectLayout L = select_layout(args, bits == nullptr);
  if (!workspace || workspace_bytes < L.total) return KVCRUSH_ERR_WORKSPACE;

  hipStream_t stream = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  const int B = args->B, Hs = args->Hs, S = args->S;
  const int Br = args->budget - args->n_important, N = S - args->n_important;
  const int kbit = args->bit_topk == 0 ? args->budget : args->bit_topk;
  uint64_t* rowmask = (uint64_t*)(ws + L.rowmask);
  uint64_t* repmask = (uint64_t*)(ws + L.repmask);
  int32_t* order = (int32_t*)(ws + L.order);
  uint64_t* bits_buf = bits ? bits : (uint64_t*)(ws + L.bits);

  {
    TopkParams p;
    p.scores = scores;
    p.rowmask = rowmask;
    p.keys_ws = L.keys_in_lds ? nullptr : (uint32_t*)(ws + L.keys);
    p.Hs = Hs;
    p.S = S;
    p.nw = L.nw;
    p.kbit = kbit;
    p.n_important = args->n_important;
    const size_t dyn = L.keys_in_lds ? (size_t)S * 4 : 0;
    if (dyn > 48 * 1024) {
      if (hipFuncSetAttribute((const void*)topk_mask_kernel,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn) != hipSuccess)
        return KVCRUSH_ERR_HIP;
    }
    hipLaunchKernelGGL(topk_mask_kernel, dim3(Hs + 1, B), dim3(kSelThreads), dyn, stream, p);
    if (kvc::launch_status() != KVCRUSH_OK) return KVCRUSH_ERR_HIP;
  }
  {
    GroupParams p;
    p.rowmask = rowmask;
    p.bits = bits_buf;
    p.order = order;
    p.repmask = repmask;
    p.anchor_bits = args->anchor_bits;
    p.anchor_seed = args->anchor_seed;
    p.Hs = Hs;
    p.S = S;
    p.nw = L.nw;
    p.W = L.W;
    p.N = N;
    p.anchor_mode = args->anchor;
    int dbits = 0;
    while ((1 << dbits) <= Hs) ++dbits;  // distances range over 0..Hs
    p.dbits = dbits;
    hipLaunchKernelGGL(group_sort_kernel, dim3(B), dim3(kSelThreads), 0, stream, p);
    if (kvc::launch_status() != KVCRUSH_OK) return KVCRUSH_ERR_HIP;
  }
  if (Br > 0) {
    MedoidParams p;
    p.bits = bits_buf;
    p.order = order;
    p.repmask = repmask;
    p.Hs = Hs;
    p.S = S;
    p.nw = L.nw;
    p.W = L.W;
    p.N = N;
    p.Br = Br;
    hipLaunchKernelGGL(medoid_kernel, dim3((Br + kMedoidWaves - 1) / kMedoidWaves, B),
                       dim3(kMedoidThreads), 0, stream, p);
    if (kvc::launch_status() != KVCRUSH_OK) return KVCRUSH_ERR_HIP;
  }
  if (args->budget > 0) {
    EmitParams p;
    p.impmask_base = rowmask + (size_t)Hs * L.nw;
    p.repmask = repmask;
    p.idx = idx;
    p.kind = kind;
    p.imp_stride = (size_t)(Hs + 1) * L.nw;
    p.S = S;
    p.nw = L.nw;
    p.budget = args->budget;
    hipLaunchKernelGGL(emit_kernel, dim3(B), dim3(kSelThreads), 0, stream, p);
    if (kvc::launch_status() != KVCRUSH_OK) return KVCRUSH_ERR_HIP;
  }
  return KVCRUSH_OK;
}
