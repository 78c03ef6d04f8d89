// Stage 1 of the KVCrush step on gfx950: the attention every cached token
// receives, per head (Alg. 1's attention weights A_h = softmax(Q_h K_h^T /
// sqrt(d_k)), accumulated over the queries as H2O does, Sec. 2.3 / 4.1.1),
// without ever writing the S x S matrix.
//
// A column sum of a row-normalised matrix needs every row's normaliser first,
// so the work is two sweeps over the causal half of Q K^T:
//
//   pass A (lse_kernel)     per query row i: lse_i = log sum_j exp(s_ij)
//                           (skipped when the caller already has it)
//   pass B (colsum_kernel)  per key t: sum_i exp(s_it - lse_i)
//
// Both compute the same 32x32 tiles  C[key][query] = K_tile . Q_tile^T  with
// v_mfma_f32_32x32x16_bf16 (fp32 inputs: v_mfma_f32_32x32x2_f32); in the MFMA
// result layout a lane owns one query column and 16 key rows, so
//   * pass A reduces over keys inside a lane (online max / sum per query),
//   * pass B subtracts a per-lane lse and adds tiles element-wise; the
//     cross-lane reduction over queries happens once, at the very end.
// The operand that stays fixed for a workgroup's lifetime (64 query rows per
// wave in pass A, 64 key rows per wave in pass B) lives in registers; the other
// one streams through double-buffered LDS tiles shared by the four waves.
// The k-index permutation inside an MFMA step is free as long as both operands
// use the same one, which lets every lane fetch its 8 (bf16) or 4 (fp32)
// contiguous elements with a single 16-byte load.
#include "common.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / KVC_WAVE;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <bool BF16, int D>
struct Cfg {
  static constexpr int kRowBytes = D * (BF16 ? 2 : 4);
  static constexpr int kSteps = kRowBytes / 32;        // 16-byte fragments per lane and row
  static constexpr int kLdsStride = kRowBytes + 16;    // pad: 16 consecutive rows hit 64 banks
  static constexpr int kTile = BF16 ? 64 : 32;         // streamed rows per LDS buffer
  static constexpr int kTileSub = kTile / 32;
  static constexpr int kChunksPerRow = kRowBytes / 16;
  static constexpr int kStage = kTile * kChunksPerRow / kThreads;  // 16-byte chunks per thread
  static constexpr int kLdsBytes = kTile * kLdsStride;
  static_assert(kTile * kChunksPerRow % kThreads == 0, "tile must split evenly over the threads");
};

// One MFMA "load step": C += A_frag . B_frag^T over this step's k-slice.
template <bool BF16>
__device__ __forceinline__ void mma_step(f32x16& acc, const u32x4& a, const u32x4& b) {
  if constexpr (BF16) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                  __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[i]), __uint_as_float(b[i]), acc,
                                                 0, 0, 0);
  }
}

// Row of the 32x32 result that register r of this lane holds.
__device__ __forceinline__ int acc_row(int r, int lane) {
  return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
}

template <class C>
__device__ __forceinline__ void stage_load(u32x4 (&st)[C::kStage], const char* head_base, int row0,
                                           int S, int tid) {
#pragma unroll
  for (int i = 0; i < C::kStage; ++i) {
    const int c = tid + kThreads * i;
    const int row = c / C::kChunksPerRow, col = c % C::kChunksPerRow;
    const int t = row0 + row;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (t < S) v = *(const u32x4*)(head_base + (size_t)t * C::kRowBytes + col * 16);
    st[i] = v;
  }
}

template <class C>
__device__ __forceinline__ void stage_store(const u32x4 (&st)[C::kStage], char* buf, int tid) {
#pragma unroll
  for (int i = 0; i < C::kStage; ++i) {
    const int c = tid + kThreads * i;
    const int row = c / C::kChunksPerRow, col = c % C::kChunksPerRow;
    *(u32x4*)(buf + row * C::kLdsStride + col * 16) = st[i];
  }
}

// Fragments of 32 stationary rows, straight from global memory to registers.
template <class C>
__device__ __forceinline__ void load_stationary(u32x4 (&frag)[C::kSteps], const char* head_base,
                                                int row0, int S, int lane) {
  const int t = row0 + (lane & 31);
#pragma unroll
  for (int s = 0; s < C::kSteps; ++s) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (t < S) v = *(const u32x4*)(head_base + (size_t)t * C::kRowBytes + s * 32 + (lane >> 5) * 16);
    frag[s] = v;
  }
}

template <class C>
__device__ __forceinline__ u32x4 lds_frag(const char* buf, int sub, int step, int lane) {
  return *(const u32x4*)(buf + (sub * 32 + (lane & 31)) * C::kLdsStride + step * 32 + (lane >> 5) * 16);
}

struct ScoreParams {
  const char* q;     // [B,Hq,S,D]
  const char* k;     // [B,Hkv,S,D]
  float* lse;        // [B,Hq,S] natural log (written by pass A, read by pass B)
  float* scores;     // [B,Hs,S]
  int B, Hq, Hkv, S, G;
  int reduce_groups;
  int heads_per_wg;  // pass A: query heads sharing one workgroup's K stream (1, 2 or 4)
  int n_blocks;      // blocks along the sequence
  int n_bh;          // (batch, head-group) pairs
  float scale_log2;  // log2(e) / sqrt(D)
};

// ------------------------------------------------------------- pass A ------
// Workgroup = 4 waves sharing one stream of K tiles.  Each wave keeps 64 query
// rows of one head in registers (two 32-row sub-tiles).  With grouped-query
// attention the waves take different heads of the same KV group (same query
// range); otherwise they take consecutive 64-row query blocks of one head.
template <bool BF16, int D>
__global__ __launch_bounds__(kThreads, 2) void lse_kernel(ScoreParams p) {
  using C = Cfg<BF16, D>;
  __shared__ __attribute__((aligned(16))) char lds[2][C::kLdsBytes];

  const int tid = threadIdx.x, lane = kvc::lane_id(), wave = tid / KVC_WAVE;
  const int S = p.S;
  // heavy (late) query blocks first; same head group -> same blockIdx residue
  const int blk = p.n_blocks - 1 - (int)(blockIdx.x / p.n_bh);
  const int bh = (int)(blockIdx.x % p.n_bh);
  const int hpw = p.heads_per_wg, qsub = kWaves / hpw;
  const int groups_per_b = p.Hq / hpw;
  const int b = bh / groups_per_b, hg = bh % groups_per_b;
  const int head = hg * hpw + wave % hpw;
  const int kvh = head / p.G;
  const int wg_q0 = blk * 64 * qsub;
  const int q0 = wg_q0 + (wave / hpw) * 64;  // first query row of this wave

  const char* qh = p.q + ((size_t)b * p.Hq + head) * S * C::kRowBytes;
  const char* kh = p.k + ((size_t)b * p.Hkv + kvh) * S * C::kRowBytes;

  u32x4 qf[2][C::kSteps];
  load_stationary<C>(qf[0], qh, q0, S, lane);
  load_stationary<C>(qf[1], qh, q0 + 32, S, lane);

  const int wg_qmax = min(S, wg_q0 + 64 * qsub) - 1;
  const int n_tiles = wg_qmax / C::kTile + 1;

  float m[2] = {-INFINITY, -INFINITY}, l[2] = {0.0f, 0.0f};
  const float c = p.scale_log2;

  u32x4 st[C::kStage];
  stage_load<C>(st, kh, 0, S, tid);
  stage_store<C>(st, lds[0], tid);
  __syncthreads();

  for (int it = 0; it < n_tiles; ++it) {
    const int kt = it * C::kTile;
    const char* buf = lds[it & 1];
    if (it + 1 < n_tiles) stage_load<C>(st, kh, kt + C::kTile, S, tid);

#pragma unroll
    for (int ks = 0; ks < C::kTileSub; ++ks) {
      const int kmin = kt + 32 * ks, kmax = kmin + 31;
      if (kmin > q0 + 63) continue;  // every key of this sub-tile is in the future of all 64 rows
      f32x16 acc[2];
#pragma unroll
      for (int ns = 0; ns < 2; ++ns)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[ns][r] = 0.0f;
#pragma unroll
      for (int s = 0; s < C::kSteps; ++s) {
        const u32x4 a = lds_frag<C>(buf, ks, s, lane);
        mma_step<BF16>(acc[0], a, qf[0][s]);
        mma_step<BF16>(acc[1], a, qf[1][s]);
      }
#pragma unroll
      for (int ns = 0; ns < 2; ++ns) {
        const int qmin = q0 + 32 * ns;
        if (kmin > qmin + 31) continue;  // uniform: nothing visible for this sub-tile
        if (kmax > qmin) {               // diagonal sub-tile: hide keys after the query
          const int lim = qmin + (lane & 31) - kmin - 4 * (lane >> 5);
#pragma unroll
          for (int r = 0; r < 16; ++r)
            acc[ns][r] = (8 * (r >> 2) + (r & 3)) <= lim ? acc[ns][r] : -INFINITY;
        }
        float mx = acc[ns][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, acc[ns][r]);
        const float mnew = fmaxf(m[ns], mx * c);
        if (mnew > -INFINITY) {
          float sum = 0.0f;
#pragma unroll
          for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[ns][r], c, -mnew));
          l[ns] = l[ns] * __builtin_amdgcn_exp2f(m[ns] - mnew) + sum;
          m[ns] = mnew;
        }
      }
    }

    if (it + 1 < n_tiles) stage_store<C>(st, lds[(it + 1) & 1], tid);
    __syncthreads();
  }

  // lanes l and l^32 saw disjoint key rows of the same query: merge, then store
#pragma unroll
  for (int ns = 0; ns < 2; ++ns) {
    const float mo = __shfl_xor(m[ns], 32), lo = __shfl_xor(l[ns], 32);
    const float mt = fmaxf(m[ns], mo);
    float lt = 0.0f;
    if (m[ns] > -INFINITY) lt += l[ns] * __builtin_amdgcn_exp2f(m[ns] - mt);
    if (mo > -INFINITY) lt += lo * __builtin_amdgcn_exp2f(mo - mt);
    const int qi = q0 + 32 * ns + (lane & 31);
    if (lane < 32 && qi < S)
      p.lse[((size_t)b * p.Hq + head) * S + qi] = (mt + __builtin_amdgcn_logf(lt)) * kLn2;
  }
}

// ------------------------------------------------------------- pass B ------
// Workgroup = 4 waves sharing one stream of Q tiles (and their lse).  Each wave
// keeps 64 key rows in registers and 2x16 running column sums; the workgroup
// covers 256 consecutive keys of one KV head and walks the query tiles from
// the end of the sequence down to its own diagonal, for one query head or,
// when the group is reduced, for each head of the group in turn.
template <bool BF16, int D>
__global__ __launch_bounds__(kThreads, 2) void colsum_kernel(ScoreParams p, const float* lse_in) {
  using C = Cfg<BF16, D>;
  __shared__ __attribute__((aligned(16))) char lds[2][C::kLdsBytes];
  __shared__ float lds_lse[2][C::kTile];

  const int tid = threadIdx.x, lane = kvc::lane_id(), wave = tid / KVC_WAVE;
  const int S = p.S;
  const int blk = (int)(blockIdx.x / p.n_bh);  // key block, early (heavy) blocks first
  const int bh = (int)(blockIdx.x % p.n_bh);
  const int rows = p.reduce_groups ? p.Hkv : p.Hq;
  const int b = bh / rows, row = bh % rows;
  const int kvh = p.reduce_groups ? row : row / p.G;
  const int head0 = p.reduce_groups ? row * p.G : row;
  const int n_heads = p.reduce_groups ? p.G : 1;
  const int wg_k0 = blk * 64 * kWaves;
  const int k0 = wg_k0 + wave * 64;  // first key row of this wave

  const char* kh = p.k + ((size_t)b * p.Hkv + kvh) * S * C::kRowBytes;
  u32x4 kf[2][C::kSteps];
  load_stationary<C>(kf[0], kh, k0, S, lane);
  load_stationary<C>(kf[1], kh, k0 + 32, S, lane);

  const int tile_lo = wg_k0 / C::kTile, tile_hi = (S - 1) / C::kTile;  // inclusive
  const int tiles_per_head = tile_hi - tile_lo + 1;
  const int n_iter = tiles_per_head * n_heads;
  const float c = p.scale_log2;

  f32x16 col[2];
#pragma unroll
  for (int ms = 0; ms < 2; ++ms)
#pragma unroll
    for (int r = 0; r < 16; ++r) col[ms][r] = 0.0f;

  auto tile_of = [&](int it, int& head, int& qt) {
    head = head0 + it / tiles_per_head;
    qt = (tile_hi - it % tiles_per_head) * C::kTile;
  };
  auto load_lse = [&](int head, int qt) -> float {
    // +inf for rows past the end makes their probabilities exactly zero
    float v = INFINITY;
    if (tid < C::kTile && qt + tid < S) v = lse_in[((size_t)b * p.Hq + head) * S + qt + tid] * kLog2e;
    return v;
  };

  u32x4 st[C::kStage];
  float st_lse;
  {
    int head, qt;
    tile_of(0, head, qt);
    stage_load<C>(st, p.q + ((size_t)b * p.Hq + head) * S * C::kRowBytes, qt, S, tid);
    st_lse = load_lse(head, qt);
    stage_store<C>(st, lds[0], tid);
    if (tid < C::kTile) lds_lse[0][tid] = st_lse;
  }
  __syncthreads();

  for (int it = 0; it < n_iter; ++it) {
    int head, qt;
    tile_of(it, head, qt);
    const char* buf = lds[it & 1];
    if (it + 1 < n_iter) {
      int nh, nqt;
      tile_of(it + 1, nh, nqt);
      stage_load<C>(st, p.q + ((size_t)b * p.Hq + nh) * S * C::kRowBytes, nqt, S, tid);
      st_lse = load_lse(nh, nqt);
    }

#pragma unroll
    for (int ns = 0; ns < C::kTileSub; ++ns) {
      const int qmin = qt + 32 * ns, qmax = qmin + 31;
      if (qmax < k0) continue;  // all 64 keys of this wave are in the future of these queries
      const float lse2 = lds_lse[it & 1][32 * ns + (lane & 31)];
      f32x16 acc[2];
#pragma unroll
      for (int ms = 0; ms < 2; ++ms)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[ms][r] = 0.0f;
#pragma unroll
      for (int s = 0; s < C::kSteps; ++s) {
        const u32x4 bq = lds_frag<C>(buf, ns, s, lane);
        mma_step<BF16>(acc[0], kf[0][s], bq);
        mma_step<BF16>(acc[1], kf[1][s], bq);
      }
#pragma unroll
      for (int ms = 0; ms < 2; ++ms) {
        const int kmin = k0 + 32 * ms;
        if (qmax < kmin) continue;
        if (kmin + 31 > qmin) {  // diagonal sub-tile
          const int lim = qmin + (lane & 31) - kmin - 4 * (lane >> 5);
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[ms][r], c, -lse2));
            col[ms][r] += (8 * (r >> 2) + (r & 3)) <= lim ? e : 0.0f;
          }
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r)
            col[ms][r] += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[ms][r], c, -lse2));
        }
      }
    }

    if (it + 1 < n_iter) {
      stage_store<C>(st, lds[(it + 1) & 1], tid);
      if (tid < C::kTile) lds_lse[(it + 1) & 1][tid] = st_lse;
    }
    __syncthreads();
  }

  // sum over the 32 query lanes of each half-wave; lanes 0 and 32 then hold the rows
  float* out = p.scores + ((size_t)b * rows + row) * S;
#pragma unroll
  for (int ms = 0; ms < 2; ++ms) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float v = col[ms][r];
#pragma unroll
      for (int off = 16; off > 0; off >>= 1) v += __shfl_xor(v, off);
      const int t = k0 + 32 * ms + acc_row(r, lane);
      if ((lane & 31) == 0 && t < S) out[t] = v;
    }
  }
}

template <bool BF16, int D>
kvcrush_status launch_lse(const ScoreParams& base, hipStream_t stream) {
  ScoreParams a = base;
  a.heads_per_wg = (a.G % 4 == 0) ? 4 : (a.G % 2 == 0 ? 2 : 1);
  const int qsub = kWaves / a.heads_per_wg;
  a.n_blocks = (a.S + 64 * qsub - 1) / (64 * qsub);
  a.n_bh = a.B * (a.Hq / a.heads_per_wg);
  hipLaunchKernelGGL((lse_kernel<BF16, D>), dim3((unsigned)(a.n_blocks * a.n_bh)), dim3(kThreads), 0,
                     stream, a);
  return kvc::launch_status();
}

template <bool BF16, int D>
kvcrush_status launch_scores(const ScoreParams& base, const float* lse_user, bool lse_only,
                             hipStream_t stream) {
  ScoreParams p = base;
  const int S = p.S;
  if (!lse_user) {
    if (launch_lse<BF16, D>(p, stream) != KVCRUSH_OK) return KVCRUSH_ERR_HIP;
  }
  if (lse_only) return KVCRUSH_OK;
  p.n_blocks = (S + 64 * kWaves - 1) / (64 * kWaves);
  p.n_bh = p.B * (p.reduce_groups ? p.Hkv : p.Hq);
  hipLaunchKernelGGL((colsum_kernel<BF16, D>), dim3((unsigned)(p.n_blocks * p.n_bh)), dim3(kThreads),
                     0, stream, p, lse_user ? lse_user : p.lse);
  return kvc::launch_status();
}

bool shape_ok(const kvcrush_shape* s) {
  if (!s) return false;
  if (s->B < 1 || s->Hq < 1 || s->Hkv < 1 || s->S < 1 || s->D < 1) return false;
  if (s->Hq % s->Hkv != 0) return false;
  if (s->dtype != KVCRUSH_F32 && s->dtype != KVCRUSH_BF16) return false;
  if (s->reduce_groups != 0 && s->reduce_groups != 1) return false;
  return true;
}

}  // namespace

extern "C" size_t kvcrush_scores_workspace(const kvcrush_shape* shape) {
  if (!shape_ok(shape)) return 0;
  return kvc::align_up((size_t)shape->B * shape->Hq * shape->S * sizeof(float), 256);
}

namespace {

kvcrush_status scores_entry(const kvcrush_shape* shape, const void* q, const void* k,
                            const float* lse, float* lse_out, float* scores, bool lse_only,
                            hipStream_t stream) {
  const long long blocks_a = (long long)shape->B * shape->Hq * ((shape->S + 63) / 64);
  if (blocks_a > 0x7FFFFFFFll) return KVCRUSH_ERR_UNSUPPORTED;
  ScoreParams p;
  p.q = (const char*)q;
  p.k = (const char*)k;
  p.lse = lse_out;
  p.scores = scores;
  p.B = shape->B;
  p.Hq = shape->Hq;
  p.Hkv = shape->Hkv;
  p.S = shape->S;
  p.G = shape->Hq / shape->Hkv;
  p.reduce_groups = shape->reduce_groups;
  p.heads_per_wg = 1;
  p.n_blocks = 0;
  p.n_bh = 0;
  p.scale_log2 = (float)(1.4426950408889634 / sqrt((double)shape->D));
  const bool bf16 = shape->dtype == KVCRUSH_BF16;
  if (bf16 && shape->D == 128) return launch_scores<true, 128>(p, lse, lse_only, stream);
  if (bf16 && shape->D == 64) return launch_scores<true, 64>(p, lse, lse_only, stream);
  if (!bf16 && shape->D == 128) return launch_scores<false, 128>(p, lse, lse_only, stream);
  return launch_scores<false, 64>(p, lse, lse_only, stream);
}

}  // namespace

extern "C" kvcrush_status kvcrush_scores(const kvcrush_shape* shape, const void* q, const void* k,
                                         const float* lse, float* scores, void* workspace,
                                         size_t workspace_bytes, void* hip_stream) {
  if (!shape_ok(shape)) return KVCRUSH_ERR_INVALID_ARG;
  if (shape->D != 64 && shape->D != 128) return KVCRUSH_ERR_UNSUPPORTED;
  if (!q || !k || !scores) return KVCRUSH_ERR_INVALID_ARG;
  if (!kvc::aligned16(q) || !kvc::aligned16(k) || !kvc::aligned16(scores) || !kvc::aligned16(lse))
    return KVCRUSH_ERR_INVALID_ARG;
  if (!lse) {
    if (!workspace || !kvc::aligned16(workspace) ||
        workspace_bytes < kvcrush_scores_workspace(shape))
      return KVCRUSH_ERR_WORKSPACE;
  }
  return scores_entry(shape, q, k, lse, (float*)workspace, scores, false, (hipStream_t)hip_stream);
}

extern "C" kvcrush_status kvcrush_row_lse(const kvcrush_shape* shape, const void* q, const void* k,
                                          float* lse_out, void* hip_stream) {
  if (!shape_ok(shape)) return KVCRUSH_ERR_INVALID_ARG;
  if (shape->D != 64 && shape->D != 128) return KVCRUSH_ERR_UNSUPPORTED;
  if (!q || !k || !lse_out) return KVCRUSH_ERR_INVALID_ARG;
  if (!kvc::aligned16(q) || !kvc::aligned16(k) || !kvc::aligned16(lse_out))
    return KVCRUSH_ERR_INVALID_ARG;
  return scores_entry(shape, q, k, nullptr, lse_out, nullptr, true, (hipStream_t)hip_stream);
}

extern "C" const char* kvcrush_status_string(kvcrush_status status) {
  switch (status) {
    case KVCRUSH_OK: return "ok";
    case KVCRUSH_ERR_INVALID_ARG: return "invalid argument";
    case KVCRUSH_ERR_UNSUPPORTED: return "unsupported configuration";
    case KVCRUSH_ERR_WORKSPACE: return "workspace missing or too small";
    case KVCRUSH_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

extern "C" int32_t kvcrush_version(void) { return 100; }
