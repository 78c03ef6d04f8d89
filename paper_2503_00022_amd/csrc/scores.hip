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
// one streams through LDS tiles shared by the four waves.
//
// Data movement.  Tiles go from global memory straight into LDS
// (global_load_lds_dwordx4, no register staging) one whole iteration ahead of
// their use, through three rotating buffers; rows are stored unpadded and the 16-byte chunks of every 256-byte
// line are XOR-swizzled by the line number, which keeps the ds_read_b128
// fragment reads free of bank conflicts.  The k-index permutation inside an
// MFMA step is free as long as both operands use the same one: lane group g
// (lane / 32) takes chunk  step + g * steps  of a row, i.e. one 16-byte load.
//
// Launch shapes.  Pass A numbers its query blocks from the end of the sequence,
// so an observation window (only the last W queries score the tokens, the
// scoring of the SnapKV baseline, Sec. 2.3) simply launches fewer of them; when
// that leaves the chip short of workgroups, the unmasked key tiles of a block
// are cut into slices, one workgroup each, and lse_combine_kernel merges the
// slices' sums.  Pass B cuts the causal triangle into pieces of equal size.
//
// Instruction order.  Away from the diagonal the bf16 kernels run a software
// pipeline written out by hand: every pair of MFMAs of the current 64x32 block
// is followed by the ds_read that fetches the same fragment of the NEXT block
// (so LDS latency is hidden behind a whole block of work) and by a slice of the
// exp / max / sum work on the PREVIOUS block's accumulators (so the matrix core
// and the VALU run side by side inside one wave).
#include <algorithm>

#include "common.h"
#include "tiles.h"

namespace {

using namespace kvc::tiles;

constexpr int kKeysPerWg = 64 * kWaves;  // pass B: keys held by one workgroup

struct ScoreParams {
  const char* q;     // row (b, h, s) at q + b * q_sb + h * q_sh + s * q_rb bytes, D values contiguous
  const char* k;     // the same with k_sb, k_sh, k_rb
  long long q_sb, q_sh, k_sb, k_sh;  // byte strides between sequences and between heads
  unsigned q_rb, k_rb;               // byte strides between consecutive tokens of one head
  bool strided;                      // false: both arrays are packed [B,H,S,D] (the strides are not read)
  float* lse;        // [B,Hq,S] natural log (written by pass A, read by pass B)
  float* scores;     // [B,Hs,S]
  float* partial;    // pass B: [n_bh, n_kb, n_chunks, 256] partial column sums (n_chunks > 1)
  int B, Hq, Hkv, S, G;
  int reduce_groups;
  int heads_per_wg;  // pass A: query heads sharing one workgroup's K stream (1, 2 or 4)
  int n_blocks;      // pass A: query blocks; pass B: 256-key blocks
  int n_bh;          // (batch, head-group) pairs
  int chunk_tiles;   // pass B: query tiles per work piece
  int n_chunks;      // pass B: chunks along the query axis
  int n_split;       // pass A: key slices per query block (1: the block's workgroup sees all its keys)
  int split_q0;      // pass A, n_split > 1: first query row held by split_ml
  int split_rows;    // pass A, n_split > 1: query rows held per head (S - split_q0)
  float2* split_ml;  // pass A, n_split > 1: [B*Hq, n_split, split_rows] (reference, sum) pairs
  int q_first;       // first query row that contributes (0 unless an observation window is set)
  int tile0;         // pass B: q_first / kTile, the first query tile that is streamed
  float scale_log2;  // log2(e) x softmax scale (1 / sqrt(D) unless the caller set one)
};

__device__ __forceinline__ void zero_acc(f32x16 (&acc)[2]) {
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
}

// Two 32x32 tiles of one block, fragments read from LDS on the spot (used off
// the fast path).  STREAM_IS_A: the LDS sub-tile supplies the rows (keys) and
// the two register operands the columns (pass A); otherwise the register
// operands supply the rows (keys) and the LDS sub-tile the columns (pass B).
template <class C, bool BF16, bool STREAM_IS_A, bool F16 = false>
__device__ __forceinline__ void mma_pair(f32x16 (&acc)[2], const char* buf, int off0, int sub,
                                         const u32x4 (&r0)[C::kSteps], const u32x4 (&r1)[C::kSteps]) {
  zero_acc(acc);
#pragma unroll
  for (int s = 0; s < C::kSteps; ++s) {
    const u32x4 f = lds_frag<C>(buf, off0, sub, s);
    if constexpr (STREAM_IS_A) {
      mma_step<BF16, F16>(acc[0], f, r0[s]);
      mma_step<BF16, F16>(acc[1], f, r1[s]);
    } else {
      mma_step<BF16, F16>(acc[0], r0[s], f);
      mma_step<BF16, F16>(acc[1], r1[s], f);
    }
  }
}

// Online max / sum over the 16 key rows a lane holds of one tile (pass A).
// With MASK, rows with 8*(r/4)+(r%4) > lim are keys after the query: left out.
template <bool MASK>
__device__ __forceinline__ void softmax_update(f32x16& acc, float& m, float& l, float c, int lim) {
  if constexpr (MASK) {
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = (8 * (r >> 2) + (r & 3)) <= lim ? acc[r] : -INFINITY;
  }
  float mx = acc[0];
#pragma unroll
  for (int r = 1; r < 16; ++r) mx = fmaxf(mx, acc[r]);
  const float mnew = fmaxf(m, mx * c);
  float sum = 0.0f;
#pragma unroll
  for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r], c, -mnew));
  l = l * __builtin_amdgcn_exp2f(m - mnew) + sum;
  m = mnew;
}

// Probabilities of one tile added to the running column sums (pass B).
template <bool MASK>
__device__ __forceinline__ void colsum_update(const f32x16& acc, f32x16& col, float c, float lse2,
                                              int lim) {
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r], c, -lse2));
    if constexpr (MASK)
      col[r] += (8 * (r >> 2) + (r & 3)) <= lim ? e : 0.0f;
    else
      col[r] += e;
  }
}

// sched_group_barrier classes: matrix ops, LDS reads, vector ALU incl. transcendentals
constexpr int kSchedMfma = 0x008, kSchedDsRead = 0x100, kSchedValu = 0x002 | 0x400;

// ---- hand-pipelined half steps (bf16, 8 fragments a block) -----------------
// acc_new = block whose fragments sit in fr[]; after each MFMA pair the same
// fragment slot is refilled from `next` (the block after it) and a slice of the
// VALU work on acc_old (the block before it) is issued.

// Fragment ring: kSteps / 2 slots.  Slot s % ring holds fragment s of the block
// being multiplied; once used it is refilled with fragment s + ring of the same
// block (first half of the steps) or fragment s - ring of the next block.
// CUR / NEXT are compile-time byte offsets of those blocks from the LDS base and
// fo[s] the lane's offset of fragment s inside a block, so that every read is
// "register + immediate" and costs no address arithmetic.
template <class C, int CUR, int NEXT>
__device__ __forceinline__ void ring_refill(u32x4 (&fr)[C::kSteps / 2], int s, const char* lds_base,
                                            const int (&fo)[C::kSteps]) {
  constexpr int kRing = C::kSteps / 2;
  if (s < kRing)
    fr[s] = *(const u32x4*)(lds_base + CUR + fo[s + kRing]);
  else
    fr[s - kRing] = *(const u32x4*)(lds_base + NEXT + fo[s - kRing]);
}

// pass B slice: 32 / kSteps of the 32 elements of acc_old per MFMA pair.
template <class C, int CUR, int NEXT, bool F16>
__device__ __forceinline__ void colsum_half(f32x16 (&acc_new)[2], const f32x16 (&acc_old)[2],
                                            f32x16 (&col)[2], u32x4 (&fr)[C::kSteps / 2],
                                            const u32x4 (&kf0)[C::kSteps], const u32x4 (&kf1)[C::kSteps],
                                            const char* lds_base, const int (&fo)[C::kSteps], float c,
                                            float lse_old) {
  constexpr int kRing = C::kSteps / 2;
  constexpr int kPer = 32 / C::kSteps;  // elements of acc_old handled per MFMA pair
  zero_acc(acc_new);
#pragma unroll
  for (int s = 0; s < C::kSteps; ++s) {
    mma_step<true, F16>(acc_new[0], kf0[s], fr[s % kRing]);
    mma_step<true, F16>(acc_new[1], kf1[s], fr[s % kRing]);
    ring_refill<C, CUR, NEXT>(fr, s, lds_base, fo);
#pragma unroll
    for (int e = s * kPer; e < (s + 1) * kPer; ++e) {
      const int t = e >> 4, r = e & 15;
      col[t][r] += __builtin_amdgcn_exp2f(__builtin_fmaf(acc_old[t][r], c, -lse_old));
    }
  }
  // issue order for the machine scheduler: every MFMA is followed by half a slice of the exp
  // work (fma, exp, add per element), the second of a pair also by the pair's refill read
  // (an MFMA right behind another holds the wave's vector instructions back until it has issued)
#pragma unroll
  for (int s = 0; s < C::kSteps; ++s) {
    __builtin_amdgcn_sched_group_barrier(kSchedMfma, 1, 0);
    __builtin_amdgcn_sched_group_barrier(kSchedValu, 3 * kPer / 2, 0);
    __builtin_amdgcn_sched_group_barrier(kSchedMfma, 1, 0);
    __builtin_amdgcn_sched_group_barrier(kSchedDsRead, 1, 0);
    __builtin_amdgcn_sched_group_barrier(kSchedValu, 3 * kPer / 2 + 1, 0);
  }
}

// pass A slice: exponentials against the lane's fixed reference m (no running
// maximum: fp32 has the range for any sum whose terms stay below 2^100 or so;
// the caller checks the sums and re-bases m in the rare case they do not).
template <class C, int CUR, int NEXT, bool F16>
__device__ __forceinline__ void lse_half(f32x16 (&acc_new)[2], const f32x16 (&acc_old)[2],
                                         const float (&m)[2], float (&sum)[2], u32x4 (&fr)[C::kSteps / 2],
                                         const u32x4 (&qf0)[C::kSteps], const u32x4 (&qf1)[C::kSteps],
                                         const char* lds_base, const int (&fo)[C::kSteps], float c) {
  constexpr int kRing = C::kSteps / 2;
  constexpr int kPer = 32 / C::kSteps;
  zero_acc(acc_new);
  sum[0] = sum[1] = 0.0f;
#pragma unroll
  for (int s = 0; s < C::kSteps; ++s) {
    mma_step<true, F16>(acc_new[0], fr[s % kRing], qf0[s]);
    mma_step<true, F16>(acc_new[1], fr[s % kRing], qf1[s]);
    ring_refill<C, CUR, NEXT>(fr, s, lds_base, fo);
#pragma unroll
    for (int e = s * kPer; e < (s + 1) * kPer; ++e) {
      const int t = e >> 4, r = e & 15;
      sum[t] += __builtin_amdgcn_exp2f(__builtin_fmaf(acc_old[t][r], c, -m[t]));
    }
  }
#pragma unroll
  for (int s = 0; s < C::kSteps; ++s) {
    __builtin_amdgcn_sched_group_barrier(kSchedMfma, 1, 0);
    __builtin_amdgcn_sched_group_barrier(kSchedValu, 3 * kPer / 2, 0);
    __builtin_amdgcn_sched_group_barrier(kSchedMfma, 1, 0);
    __builtin_amdgcn_sched_group_barrier(kSchedDsRead, 1, 0);
    __builtin_amdgcn_sched_group_barrier(kSchedValu, 3 * kPer / 2 + 1, 0);
  }
}

// Adds a block's sums to the running (m, l) pair; re-bases on the block's own
// maximum when a sum left the safe range (wave-uniform, rare).
__device__ __forceinline__ void lse_commit(const f32x16 (&acc)[2], float (&m)[2], float (&l)[2],
                                           const float (&sum)[2], float c) {
  constexpr float kSafe = 1.0e30f;
  const bool bad = !(l[0] + sum[0] < kSafe) || !(l[1] + sum[1] < kSafe);
  if (__builtin_expect(__any(bad), 0)) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      f32x16 a = acc[t];
      softmax_update<false>(a, m[t], l[t], c, 0);
    }
  } else {
    l[0] += sum[0];
    l[1] += sum[1];
  }
}

template <int N>
struct IntC { static constexpr int value = N; };

// ------------------------------------------------------------- pass A ------
// Workgroup = 4 waves sharing one stream of K tiles.  Each wave keeps 64 query
// rows of one head in registers (two 32-row sub-tiles).  With grouped-query
// attention the waves take different heads of the same KV group (same query
// range); otherwise they take consecutive 64-row query blocks of one head.
// K tiles wholly before the workgroup's first query need no mask and run in the
// pipelined loop; the few tiles that touch the diagonal go through a plain
// masked loop afterwards.
// STRIDED: Q and K rows lie where the caller's strides put them; otherwise the
// packed [B,H,S,D] layout, whose strides are compile-time constants.
template <bool BF16, int D, bool F16 = false, bool STRIDED = false>
__global__ __launch_bounds__(kThreads, 2) void lse_kernel(ScoreParams p) {
  using C = Cfg<BF16, D>;
  __shared__ __attribute__((aligned(1024))) char lds[3][C::kTileBytes];

  const int tid = threadIdx.x, lane = kvc::lane_id(), wave = tid / KVC_WAVE;
  const int S = p.S;
  // heavy (late) query blocks first; same head group -> same blockIdx residue
  const int bh = (int)(blockIdx.x % p.n_bh);
  const int piece = (int)(blockIdx.x / p.n_bh);
  const int slice = piece % p.n_split;  // key slice of the unmasked tiles; the last also takes the diagonal
  const int blk = p.n_blocks - 1 - piece / p.n_split;
  const int hpw = p.heads_per_wg, qsub = kWaves / hpw;
  const int groups_per_b = p.Hq / hpw;
  const int b = bh / groups_per_b, hg = bh % groups_per_b;
  const int head = hg * hpw + wave % hpw;
  const int kvh = head / p.G;
  const int wg_q0 = blk * 64 * qsub;
  const int q0 = wg_q0 + (wave / hpw) * 64;  // first query row of this wave

  const char* qh = STRIDED ? p.q + b * p.q_sb + head * p.q_sh : p.q + ((size_t)b * p.Hq + head) * S * C::kRowBytes;
  const char* kh = STRIDED ? p.k + b * p.k_sb + kvh * p.k_sh : p.k + ((size_t)b * p.Hkv + kvh) * S * C::kRowBytes;
  const unsigned qrb = STRIDED ? p.q_rb : (unsigned)C::kRowBytes, krb = STRIDED ? p.k_rb : (unsigned)C::kRowBytes;

  u32x4 qf[2][C::kSteps];
  load_stationary<C>(qf[0], qh, q0, S, lane, qrb);
  load_stationary<C>(qf[1], qh, q0 + 32, S, lane, qrb);

  const int wg_qmax = min(S, wg_q0 + 64 * qsub) - 1;
  const int n_tiles = wg_qmax / C::kTile + 1;
  // tiles whose keys all precede every query of the workgroup; this workgroup's
  // slice of them is [f_begin, f_begin + n_full)
  const int n_before = C::kPipelined ? wg_q0 / C::kTile : 0;
  const int f_begin = n_before * slice / p.n_split;
  const int n_full = n_before * (slice + 1) / p.n_split - f_begin;
  const int off0 = lds_frag_offset0<C>(lane);
  uint32_t rel[C::kLoadsPerWave];
  tile_lane_offsets<C>(rel, wave, lane, krb);

  float m[2] = {kNegBig, kNegBig}, l[2] = {0.0f, 0.0f};
  const float c = p.scale_log2;

  if constexpr (C::kPipelined) {
    if (n_full > 0) {
      // (these tiles end before the workgroup's first query: always whole)
      tile_load_async_full<C>(kh, f_begin * C::kTile, lds[0], rel, wave, krb);
      tile_load_async_full<C>(kh, (f_begin + min(1, n_full - 1)) * C::kTile, lds[1], rel, wave, krb);
      wait_async_loads();
      __syncthreads();
      // tile t lives in lds[t % 3]: while iteration `it` multiplies tiles it and
      // it + 1, tile it + 2 lands in the buffer tile it - 1 has left.  The loop
      // is unrolled three times so that every buffer address is an immediate.
      const char* lds_base = &lds[0][0];
      const uint32_t wave_dst = tile_wave_dst(lds_base, wave);
      const char* kh_u = wave_uniform(kh);  // (the wave's head picks it: uniform, but not to the compiler)
      int fo[C::kSteps];
#pragma unroll
      for (int s = 0; s < C::kSteps; ++s) fo[s] = off0 ^ (s << 4);
      f32x16 acc0[2], acc1[2];
      u32x4 fr[C::kSteps / 2];
      mma_pair<C, BF16, true, F16>(acc0, lds[0], off0, 0, qf[0], qf[1]);
#pragma unroll
      for (int s = 0; s < C::kSteps / 2; ++s) fr[s] = lds_frag<C>(lds[0], off0, 1, s);
      // reference for the exponentials: the first block's own maximum
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        float mx = acc0[t][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, acc0[t][r]);
        m[t] = mx * c;
      }
      // The trip count is rounded up to a multiple of three; the padding
      // iterations run on the last tile again with an infinite reference, so
      // every exponential they produce is exactly zero.
      auto body = [&](auto P, int it) {
        constexpr int cur = decltype(P)::value, nxt = (cur + 1) % 3, ld = (cur + 2) % 3;
        constexpr int kT = C::kTileBytes, kU = C::kSubBytes;
        tile_load_async_full_unseen<C>(kh_u + (size_t)((f_begin + min(it + 2, n_full - 1)) * C::kTile) * krb,
                                       wave_dst + ld * kT, rel);
        const bool live = it < n_full;
        float sum[2], mref[2];
        // block (it, sub 1) goes through the MFMAs while block (it, sub 0) is summed
        mref[0] = live ? m[0] : INFINITY;
        mref[1] = live ? m[1] : INFINITY;
        lse_half<C, cur * kT + kU, nxt * kT, F16>(acc1, acc0, mref, sum, fr, qf[0], qf[1], lds_base, fo, c);
        lse_commit(acc0, m, l, sum, c);
        mref[0] = live ? m[0] : INFINITY;
        mref[1] = live ? m[1] : INFINITY;
        lse_half<C, nxt * kT, nxt * kT + kU, F16>(acc0, acc1, mref, sum, fr, qf[0], qf[1], lds_base, fo, c);
        lse_commit(acc1, m, l, sum, c);
        wait_async_loads();
        __syncthreads();
      };
      for (int it = 0; it < n_full; it += 3) {
        body(IntC<0>{}, it);
        body(IntC<1>{}, it + 1);
        body(IntC<2>{}, it + 2);
      }
    }
  }

  if (n_tiles > n_before && slice == p.n_split - 1) {
    tile_load_async<C>(kh, n_before * C::kTile, S, lds[0], rel, wave, lane, krb);
    wait_async_loads();
    __syncthreads();
    for (int it = n_before; it < n_tiles; ++it) {
      const int kt = it * C::kTile;
      const char* buf = lds[(it - n_before) & 1];
      if (it + 1 < n_tiles) tile_load_async<C>(kh, kt + C::kTile, S, lds[(it - n_before + 1) & 1], rel, wave, lane, krb);
#pragma unroll
      for (int ks = 0; ks < C::kTileSub; ++ks) {
        const int kmin = kt + 32 * ks, kmax = kmin + 31;
        if (kmin > q0 + 63) continue;  // every key of this sub-tile comes after all 64 rows
        f32x16 acc[2];
        mma_pair<C, BF16, true, F16>(acc, buf, off0, ks, qf[0], qf[1]);
#pragma unroll
        for (int ns = 0; ns < 2; ++ns) {
          const int qmin = q0 + 32 * ns;
          if (kmin > qmin + 31) continue;  // uniform: nothing visible for this sub-tile
          if (kmax > qmin) {
            const int lim = qmin + (lane & 31) - kmin - 4 * (lane >> 5);
            softmax_update<true>(acc[ns], m[ns], l[ns], c, lim);
          } else {
            softmax_update<false>(acc[ns], m[ns], l[ns], c, 0);
          }
        }
      }
      wait_async_loads();
      __syncthreads();
    }
  }

  // lanes l and l^32 saw disjoint key rows of the same query: merge, then store
#pragma unroll
  for (int ns = 0; ns < 2; ++ns) {
    const float mo = __shfl_xor(m[ns], 32), lo = __shfl_xor(l[ns], 32);
    const float mt = fmaxf(m[ns], mo);
    const float lt = l[ns] * __builtin_amdgcn_exp2f(m[ns] - mt) + lo * __builtin_amdgcn_exp2f(mo - mt);
    const int qi = q0 + 32 * ns + (lane & 31);
    if (lane < 32 && qi < S) {
      if (p.n_split == 1)
        p.lse[((size_t)b * p.Hq + head) * S + qi] = (mt + __builtin_amdgcn_logf(lt)) * kLn2;
      else
        p.split_ml[(((size_t)b * p.Hq + head) * p.n_split + slice) * p.split_rows + (qi - p.split_q0)] =
            make_float2(mt, lt);
    }
  }
}

// lse of the rows whose keys were cut into slices: the slices' (reference, sum)
// pairs stand for sum * 2^reference.  One wave per query row, lane s holds slice
// s (there are at most 64); the sum over the slices is a fixed shuffle tree.
__global__ __launch_bounds__(256) void lse_combine_kernel(ScoreParams p) {
  const int lane = kvc::lane_id();
  const int r = blockIdx.x * (256 / KVC_WAVE) + threadIdx.x / KVC_WAVE, bh = blockIdx.y;  // bh = b * Hq + head
  if (r >= p.split_rows) return;
  float2 ml = make_float2(kNegBig, 0.0f);
  if (lane < p.n_split) ml = p.split_ml[((size_t)bh * p.n_split + lane) * p.split_rows + r];
  float mt = ml.x;
#pragma unroll
  for (int off = KVC_WAVE / 2; off > 0; off >>= 1) mt = fmaxf(mt, __shfl_xor(mt, off));
  float lt = ml.y * __builtin_amdgcn_exp2f(ml.x - mt);
#pragma unroll
  for (int off = KVC_WAVE / 2; off > 0; off >>= 1) lt += __shfl_xor(lt, off);
  if (lane == 0) p.lse[(size_t)bh * p.S + p.split_q0 + r] = (mt + __builtin_amdgcn_logf(lt)) * kLn2;
}

// ------------------------------------------------------------- pass B ------
// Workgroup = 4 waves sharing one stream of Q tiles (and their lse).  Each wave
// keeps 64 key rows in registers and 2x16 running column sums; the workgroup
// covers 256 consecutive keys of one KV head.  The causal triangle of
// (key block, query tile) pairs is cut into pieces of at most `chunk_tiles`
// query tiles so that all workgroups get similar amounts of work; pieces that
// share a query chunk are neighbours in launch order, so the Q tiles they
// stream stay in the L2 of their XCD.  A piece covers every query head of the
// score row (one head, or the whole group when groups are reduced).  When a key
// block needs more than one piece, each writes partial sums and
// colsum_reduce_kernel adds them in a fixed order (no floating-point atomics:
// the result does not depend on scheduling).
template <bool BF16, int D, bool F16 = false, bool STRIDED = false>
__global__ __launch_bounds__(kThreads, 2) void colsum_kernel(ScoreParams p, const float* lse_in) {
  using C = Cfg<BF16, D>;
  __shared__ __attribute__((aligned(1024))) char lds[3][C::kTileBytes];
  __shared__ float lds_lse[3][kThreads];  // first kTile entries of a row are used

  const int tid = threadIdx.x, lane = kvc::lane_id(), wave = tid / KVC_WAVE;
  const int S = p.S;
  constexpr int kTpk = kKeysPerWg / C::kTile;  // query tiles spanned by the workgroup's keys
  const int n_tiles = (S + C::kTile - 1) / C::kTile;
  const int n_kb = p.n_blocks;

  // piece -> (chunk, key block): chunks from the start of the sequence on.  The early chunks have
  // few key blocks and pieces of uneven length (many diagonal tiles); the late ones are a full row
  // of key blocks each, all pieces alike, and the very last chunk is the short remainder: started
  // in this order the workgroup slots of the chip run dry at nearly the same time.
  const int bh = (int)(blockIdx.x % p.n_bh);
  int rem = (int)(blockIdx.x / p.n_bh);
  int chunk = 0;
  int t_last;
  for (;;) {
    t_last = min(p.tile0 + (chunk + 1) * p.chunk_tiles, n_tiles) - 1;
    const int cnt = min(n_kb, t_last / kTpk + 1);
    if (rem < cnt) break;
    rem -= cnt;
    ++chunk;
  }
  const int kb = rem;

  const int rows = p.reduce_groups ? p.Hkv : p.Hq;
  const int b = bh / rows, row = bh % rows;
  const int kvh = p.reduce_groups ? row : row / p.G;
  const int head0 = p.reduce_groups ? row * p.G : row;
  const int n_heads = p.reduce_groups ? p.G : 1;
  const int wg_k0 = kb * kKeysPerWg;
  const int k0 = wg_k0 + wave * 64;  // first key row of this wave

  const char* kh = STRIDED ? p.k + b * p.k_sb + kvh * p.k_sh : p.k + ((size_t)b * p.Hkv + kvh) * S * C::kRowBytes;
  const unsigned qrb = STRIDED ? p.q_rb : (unsigned)C::kRowBytes, krb = STRIDED ? p.k_rb : (unsigned)C::kRowBytes;
  u32x4 kf[2][C::kSteps];
  load_stationary<C>(kf[0], kh, k0, S, lane, krb);
  load_stationary<C>(kf[1], kh, k0 + 32, S, lane, krb);

  // tiles of this piece: [t_first, t_last]; those below f_first touch the diagonal, and the
  // sequence's last tile, when it is a partial one, is taken out of the pipelined range as well
  // (every tile there is whole, so its loads need no row clamp: fewer address instructions
  // beside the MFMAs)
  const int t_first = max(p.tile0 + chunk * p.chunk_tiles, kb * kTpk);
  const int f_first = C::kPipelined ? max(t_first, kb * kTpk + kTpk) : t_last + 1;
  const bool ragged_last = (t_last + 1) * C::kTile > S;
  const int f_last = t_last - (ragged_last ? 1 : 0);
  const int n_fullt = max(0, f_last - f_first + 1);
  const int d_last = min(f_first - 1, t_last);
  const int n_diagt = max(0, d_last - t_first + 1);
  const int n_extra = (ragged_last && t_last >= f_first) ? 1 : 0;  // the partial tile, if not among the diagonal ones
  const float c = p.scale_log2;
  const int off0 = lds_frag_offset0<C>(lane);
  uint32_t rel[C::kLoadsPerWave];
  tile_lane_offsets<C>(rel, wave, lane, qrb);

  f32x16 col[2];
  zero_acc(col);

  auto q_head = [&](int head) {
    return STRIDED ? p.q + b * p.q_sb + head * p.q_sh : p.q + ((size_t)b * p.Hq + head) * S * C::kRowBytes;
  };
  const unsigned n_live = (unsigned)(S - p.q_first);
  auto load_lse = [&](int head, int qt) -> float {
    // +inf for rows past the end makes their probabilities exactly zero.  Branch
    // free (clamped address, select) so that the caller's loop body stays one
    // straight block; threads beyond the tile re-read its rows and are ignored.
    const int i = qt + (tid & (C::kTile - 1));
    const float v = lse_in[((size_t)b * p.Hq + head) * S + min(i, S - 1)] * kLog2e;
    // one unsigned compare covers both ends: q_first <= i < S (rows before an
    // observation window contribute nothing either)
    return (unsigned)(i - p.q_first) < n_live ? v : INFINITY;
  };

  // ---- tiles after the diagonal: no mask, hand-pipelined
  if constexpr (C::kPipelined) {
    const int n_fast = n_heads * n_fullt;
    if (n_fast > 0) {
      // The (head, tile) pairs are walked with running pointers: a head's tiles from f_last down
      // to f_first, then the next head.  Steps past the last pair stay on it (their lse is +inf).
      // Scalar adds and one compare per step: no division, no 64-bit multiply inside the loop.
      const long long head_step = STRIDED ? p.q_sh : (long long)S * C::kRowBytes;  // bytes between heads
      const long long tile_step = (long long)C::kTile * qrb;                      // bytes between tiles
      const long long head_jump = head_step + (long long)(n_fullt - 1) * tile_step;
      const char* q_next = wave_uniform(q_head(head0) + (size_t)f_last * C::kTile * qrb);
      // A lane needs the lse of two query rows of a tile (lane % 32 of either 32-row block): it
      // loads them itself, two tiles ahead, and keeps them in registers.
      const float* lse_next = lse_in + ((size_t)b * p.Hq + head0) * S + (size_t)f_last * C::kTile + (lane & 31);
      int qt_next = f_last * C::kTile, left = n_fullt, pair_no = 0;
      // The loads are written out so that nothing waits for them before the end-of-step wait that
      // the tile loads need anyway: the registers hold no value until settle() has run.
      struct Pending {
        float raw[2];
        bool counts[2];
      };
      // loads pair `pair_no` (tile -> buf) and starts the loads of this lane's two lse values of it
      const uint32_t wave_dst = tile_wave_dst(&lds[0][0], wave);
      auto issue = [&](int buf_no) -> Pending {
        Pending x;
        tile_load_async_full_unseen<C>(q_next, wave_dst + buf_no * C::kTileBytes, rel);
        asm volatile("global_load_dword %0, %2, off\n\tglobal_load_dword %1, %2, off offset:128"
                     : "=&v"(x.raw[0]), "=&v"(x.raw[1])
                     : "v"(lse_next)
                     : "memory");
        // (every tile here is whole; rows before an observation window contribute nothing)
        x.counts[0] = pair_no < n_fast && qt_next + (lane & 31) >= p.q_first;
        x.counts[1] = pair_no < n_fast && qt_next + 32 + (lane & 31) >= p.q_first;
        // (selects, not branches: the loop body has to stay one straight block)
        const bool more = pair_no < n_fast - 1, wrap = left == 1;
        const long long dq = more ? (wrap ? head_jump : -tile_step) : 0ll;
        const int dl = more ? (wrap ? S + (n_fullt - 1) * C::kTile : -C::kTile) : 0;
        q_next += dq;
        lse_next += dl;
        qt_next = more ? (wrap ? f_last * C::kTile : qt_next - C::kTile) : qt_next;
        left = more ? (wrap ? n_fullt : left - 1) : left;
        ++pair_no;
        return x;
      };
      // waits for every load in flight (tiles and lse) and turns the pair's lse into base 2
      auto settle = [&](Pending& x, float (&lse2)[2]) {
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(x.raw[0]), "+v"(x.raw[1])::"memory");
        lse2[0] = x.counts[0] ? x.raw[0] * kLog2e : INFINITY;
        lse2[1] = x.counts[1] ? x.raw[1] * kLog2e : INFINITY;
      };
      float lse_cur[2], lse_nxt[2];
      {
        Pending x0 = issue(0);
        Pending x1 = issue(1);
        settle(x0, lse_cur);
        settle(x1, lse_nxt);
      }
      __syncthreads();
      // tile t lives in buffer t % 3, as in pass A
      const char* lds_base = &lds[0][0];
      int fo[C::kSteps];
#pragma unroll
      for (int s = 0; s < C::kSteps; ++s) fo[s] = off0 ^ (s << 4);
      f32x16 acc0[2], acc1[2];
      u32x4 fr[C::kSteps / 2];
      mma_pair<C, BF16, false, F16>(acc0, lds[0], off0, 0, kf[0], kf[1]);
#pragma unroll
      for (int s = 0; s < C::kSteps / 2; ++s) fr[s] = lds_frag<C>(lds[0], off0, 1, s);
      // The trip count is rounded up to a multiple of three; the padding
      // iterations run on the last tile again with lse = +inf, so every
      // probability they produce is exactly zero.
      auto body = [&](auto P, int it) {
        constexpr int cur = decltype(P)::value, nxt = (cur + 1) % 3, ld = (cur + 2) % 3;
        constexpr int kT = C::kTileBytes, kU = C::kSubBytes;
        Pending ahead = issue(ld);  // pair it + 2
        colsum_half<C, cur * kT + kU, nxt * kT, F16>(acc1, acc0, col, fr, kf[0], kf[1], lds_base, fo, c, lse_cur[0]);
        colsum_half<C, nxt * kT, nxt * kT + kU, F16>(acc0, acc1, col, fr, kf[0], kf[1], lds_base, fo, c, lse_cur[1]);
        lse_cur[0] = lse_nxt[0];
        lse_cur[1] = lse_nxt[1];
        settle(ahead, lse_nxt);
        __syncthreads();
      };
      for (int it = 0; it < n_fast; it += 3) {
        body(IntC<0>{}, it);
        body(IntC<1>{}, it + 1);
        body(IntC<2>{}, it + 2);
      }
    }
  }

  // ---- tiles on the diagonal (and every tile of the fp32 path): masked, plain loop
  const int n_slowt = n_diagt + n_extra;
  const int n_slow = n_heads * n_slowt;
  if (n_slow > 0) {
    auto tile_of = [&](int it, int& head, int& qt) {
      head = head0 + it / n_slowt;
      const int j = it % n_slowt;
      qt = (j < n_extra ? t_last : d_last - (j - n_extra)) * C::kTile;
    };
    int head, qt;
    tile_of(0, head, qt);
    tile_load_async<C>(q_head(head), qt, S, lds[0], rel, wave, lane, qrb);
    lds_lse[0][tid] = load_lse(head, qt);
    wait_async_loads();
    __syncthreads();
    for (int it = 0; it < n_slow; ++it) {
      tile_of(it, head, qt);
      const int qt_cur = qt;
      const char* buf = lds[it & 1];
      float st_lse = 0.0f;
      if (it + 1 < n_slow) {
        tile_of(it + 1, head, qt);
        tile_load_async<C>(q_head(head), qt, S, lds[(it + 1) & 1], rel, wave, lane, qrb);
        st_lse = load_lse(head, qt);
      }
#pragma unroll
      for (int ns = 0; ns < C::kTileSub; ++ns) {
        const int qmin = qt_cur + 32 * ns, qmax = qmin + 31;
        if (qmax < k0) continue;  // all 64 keys of this wave come after these queries
        const float lse2 = lds_lse[it & 1][32 * ns + (lane & 31)];
        f32x16 acc[2];
        mma_pair<C, BF16, false, F16>(acc, buf, off0, ns, kf[0], kf[1]);
#pragma unroll
        for (int ms = 0; ms < 2; ++ms) {
          const int kmin = k0 + 32 * ms;
          if (qmax < kmin) continue;
          if (kmin + 31 > qmin) {
            const int lim = qmin + (lane & 31) - kmin - 4 * (lane >> 5);
            colsum_update<true>(acc[ms], col[ms], c, lse2, lim);
          } else {
            colsum_update<false>(acc[ms], col[ms], c, lse2, 0);
          }
        }
      }
      if (it + 1 < n_slow) lds_lse[(it + 1) & 1][tid] = st_lse;
      wait_async_loads();
      __syncthreads();
    }
  }

  // sum over the 32 query lanes of each half-wave; lanes 0 and 32 then hold the rows
  float* out;
  int t_limit;
  if (p.n_chunks == 1) {
    out = p.scores + (size_t)bh * S + k0;
    t_limit = S - k0;
  } else {
    out = p.partial + (((size_t)bh * n_kb + kb) * p.n_chunks + chunk) * kKeysPerWg + wave * 64;
    t_limit = 64;
  }
#pragma unroll
  for (int ms = 0; ms < 2; ++ms) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float v = col[ms][r];
#pragma unroll
      for (int off = 16; off > 0; off >>= 1) v += __shfl_xor(v, off);
      const int t = 32 * ms + acc_row(r, lane);
      if ((lane & 31) == 0 && t < t_limit) out[t] = v;
    }
  }
}

// scores[bh, t] = sum of the partial sums of key t's pieces, chunks ascending.
__global__ __launch_bounds__(kKeysPerWg) void colsum_reduce_kernel(ScoreParams p, int tiles_per_kb) {
  const int kb = blockIdx.x, bh = blockIdx.y;
  const int t = kb * kKeysPerWg + threadIdx.x;
  if (t >= p.S) return;
  const int c_min = max(0, kb * tiles_per_kb - p.tile0) / p.chunk_tiles;
  const float* src = p.partial + ((size_t)bh * p.n_blocks + kb) * p.n_chunks * kKeysPerWg + threadIdx.x;
  float acc = 0.0f;
  int c = c_min;
  for (; c + 4 <= p.n_chunks; c += 4) {  // four loads in flight, added in chunk order
    const float x0 = src[(size_t)c * kKeysPerWg], x1 = src[(size_t)(c + 1) * kKeysPerWg];
    const float x2 = src[(size_t)(c + 2) * kKeysPerWg], x3 = src[(size_t)(c + 3) * kKeysPerWg];
    acc = (((acc + x0) + x1) + x2) + x3;
  }
  for (; c < p.n_chunks; ++c) acc += src[(size_t)c * kKeysPerWg];
  p.scores[(size_t)bh * p.S + t] = acc;
}

// Work pieces of pass B for a sequence of n_tiles query tiles.
struct ColsumPlan {
  int n_kb, n_chunks, chunk_tiles;
  long long pieces;  // per (batch, score row)
};

constexpr long long kMaxGridX = 0x7FFFFFFFll;  // workgroups of a one-dimensional launch
constexpr long long kMaxGridY = 65535;

ColsumPlan colsum_plan(int S, int tile, int chunk_tiles_wanted, int q_first) {
  ColsumPlan pl;
  const int n_tiles = (S + tile - 1) / tile, tpk = kKeysPerWg / tile, tile0 = q_first / tile;
  pl.n_kb = (S + kKeysPerWg - 1) / kKeysPerWg;
  pl.chunk_tiles = chunk_tiles_wanted;
  pl.n_chunks = (n_tiles - tile0 + pl.chunk_tiles - 1) / pl.chunk_tiles;
  pl.pieces = 0;
  for (int c = 0; c < pl.n_chunks; ++c) {
    const int end = tile0 + (c + 1) * pl.chunk_tiles;
    const int t_last = end < n_tiles ? end - 1 : n_tiles - 1;
    const int cnt = t_last / tpk + 1;
    pl.pieces += cnt < pl.n_kb ? cnt : pl.n_kb;
  }
  return pl;
}

// Pass-B work pieces run about 72 tile steps each (query tiles x the heads a piece walks): 18
// tiles of 64 queries when a score row sums a KV group of four query heads, 72 when it is one
// head.  The count is a multiple of three (the loop's unroll).
constexpr int kPieceSteps = 72;
int chunk_tiles_for(int tile, int heads_per_row) {
  const int steps = kPieceSteps * 64 / tile;                       // (fp32 tiles hold 32 queries)
  const int tiles = (steps + heads_per_row - 1) / heads_per_row;
  return std::max(3, (tiles + 2) / 3 * 3);
}

// Launch shape of pass A.  Query blocks are numbered from the end of the
// sequence: with an observation window only the blocks that reach into it are
// launched.  When that leaves the chip short of workgroups (short windows, few
// heads) and the caller gave scratch memory, the unmasked key tiles of every
// block are cut into n_split slices, one workgroup each.
struct LsePlan {
  int heads_per_wg, n_blocks, n_bh, launched, n_split, split_q0, split_rows;
};

// Two per compute unit.  (With 512 whole blocks already, slices and their merge cost more than
// they balance: 112 us against 97 us at S = 4096 with 32 heads.)
constexpr int kWantedWorkgroups = 512;
constexpr int kMinTilesPerSlice = 4;
constexpr int kMaxSplit = 64;
static_assert(kMaxSplit <= KVC_WAVE, "lse_combine_kernel gives one lane to each slice");

LsePlan lse_plan(int B, int Hq, int Hkv, int S, bool bf16, int q_first, bool may_split) {
  LsePlan pl;
  const int G = Hq / Hkv;
  pl.heads_per_wg = (G % 4 == 0) ? 4 : (G % 2 == 0 ? 2 : 1);
  const int qb = 64 * (kWaves / pl.heads_per_wg);  // query rows per workgroup
  pl.n_blocks = (S + qb - 1) / qb;
  pl.n_bh = B * (Hq / pl.heads_per_wg);
  const int first_blk = q_first / qb;
  pl.launched = pl.n_blocks - first_blk;
  pl.n_split = 1;
  pl.split_q0 = first_blk * qb;
  pl.split_rows = S - pl.split_q0;
  const long long wgs = (long long)pl.launched * pl.n_bh;
  if (may_split && bf16 && wgs < kWantedWorkgroups) {
    const int tiles_last = (pl.n_blocks - 1) * qb / 64;  // unmasked key tiles of the last block
    int n = (int)((kWantedWorkgroups + wgs - 1) / wgs);
    n = std::min(n, std::min(kMaxSplit, tiles_last / kMinTilesPerSlice));
    pl.n_split = std::max(n, 1);
  }
  return pl;
}

size_t split_bytes(const LsePlan& pl, int B, int Hq) {
  if (pl.n_split <= 1) return 0;
  return kvc::align_up((size_t)B * Hq * pl.n_split * pl.split_rows * sizeof(float2), 256);
}

template <bool BF16, int D, bool F16 = false>
kvcrush_status launch_lse(const ScoreParams& base, float2* split_ml, hipStream_t stream) {
  ScoreParams a = base;
  const LsePlan pl = lse_plan(a.B, a.Hq, a.Hkv, a.S, BF16, a.q_first, split_ml != nullptr);
  a.heads_per_wg = pl.heads_per_wg;
  a.n_blocks = pl.n_blocks;
  a.n_bh = pl.n_bh;
  a.n_split = pl.n_split;
  a.split_q0 = pl.split_q0;
  a.split_rows = pl.split_rows;
  a.split_ml = split_ml;
  if ((long long)pl.launched * pl.n_split * pl.n_bh > kMaxGridX) return KVCRUSH_ERR_UNSUPPORTED;
  const dim3 grid((unsigned)(pl.launched * pl.n_split * pl.n_bh));
  const kvcrush_status st = a.strided ? kvc::launch(lse_kernel<BF16, D, F16, true>, grid, dim3(kThreads), 0, stream, a)
                                      : kvc::launch(lse_kernel<BF16, D, F16, false>, grid, dim3(kThreads), 0, stream, a);
  if (st != KVCRUSH_OK || pl.n_split <= 1) return st;
  return kvc::launch(lse_combine_kernel, dim3((pl.split_rows + 3) / 4, a.B * a.Hq), dim3(256), 0, stream, a);
}

template <bool BF16, int D, bool F16 = false>
kvcrush_status launch_scores(const ScoreParams& base, const float* lse_user, float2* split_ml,
                             bool lse_only, hipStream_t stream) {
  using C = Cfg<BF16, D>;
  ScoreParams p = base;
  const ColsumPlan pl = colsum_plan(p.S, C::kTile, chunk_tiles_for(C::kTile, p.reduce_groups ? p.G : 1), p.q_first);
  const long long rows = (long long)p.B * (p.reduce_groups ? p.Hkv : p.Hq);
  if (!lse_only && pl.pieces * rows > kMaxGridX) return KVCRUSH_ERR_UNSUPPORTED;  // before anything is enqueued
  if (!lse_user) {
    const kvcrush_status st = launch_lse<BF16, D, F16>(p, split_ml, stream);
    if (st != KVCRUSH_OK) return st;
  }
  if (lse_only) return KVCRUSH_OK;
  p.tile0 = p.q_first / C::kTile;
  p.n_blocks = pl.n_kb;
  p.n_chunks = pl.n_chunks;
  p.chunk_tiles = pl.chunk_tiles;
  p.n_bh = p.B * (p.reduce_groups ? p.Hkv : p.Hq);
  const dim3 grid((unsigned)(pl.pieces * p.n_bh));
  const float* lse_in = lse_user ? lse_user : p.lse;
  const kvcrush_status st =
      p.strided ? kvc::launch(colsum_kernel<BF16, D, F16, true>, grid, dim3(kThreads), 0, stream, p, lse_in)
                : kvc::launch(colsum_kernel<BF16, D, F16, false>, grid, dim3(kThreads), 0, stream, p, lse_in);
  if (st != KVCRUSH_OK || pl.n_chunks <= 1) return st;
  return kvc::launch(colsum_reduce_kernel, dim3(pl.n_kb, p.n_bh), dim3(kKeysPerWg), 0, stream, p,
                     kKeysPerWg / C::kTile);
}

// First query row that contributes to the scores.
int first_query(const kvcrush_shape* s) {
  return (s->obs_window <= 0 || s->obs_window >= s->S) ? 0 : s->S - s->obs_window;
}

// Workspace: [lse: B*Hq*S floats][partial column sums]
size_t lse_bytes(const kvcrush_shape* s) {
  return kvc::align_up((size_t)s->B * s->Hq * s->S * sizeof(float), 256);
}

size_t partial_bytes(const kvcrush_shape* s) {
  const int tile = s->dtype != KVCRUSH_F32 ? 64 : 32;
  const ColsumPlan pl = colsum_plan(s->S, tile, chunk_tiles_for(tile, s->reduce_groups ? s->Hq / s->Hkv : 1), first_query(s));
  if (pl.n_chunks <= 1) return 0;
  const size_t rows = (size_t)s->B * (s->reduce_groups ? s->Hkv : s->Hq);
  return kvc::align_up(rows * pl.n_kb * pl.n_chunks * kKeysPerWg * sizeof(float), 256);
}

size_t split_bytes(const kvcrush_shape* s) {
  return split_bytes(lse_plan(s->B, s->Hq, s->Hkv, s->S, s->dtype != KVCRUSH_F32, first_query(s), true),
                     s->B, s->Hq);
}

size_t elem_bytes(const kvcrush_shape* s) { return s->dtype == KVCRUSH_F32 ? 4 : 2; }

// A caller's strides (elements): all zero (packed), or all positive, multiples of
// 16 bytes, rows not overlapping their own D values.
bool strides_ok(const int64_t (&st)[3], const kvcrush_shape* s) {
  if (st[0] == 0 && st[1] == 0 && st[2] == 0) return true;
  const long long eb = (long long)elem_bytes(s);
  for (int i = 0; i < 3; ++i) {
    if (st[i] <= 0 || st[i] > (1ll << 56) || (st[i] * eb) % 16 != 0) return false;
  }
  return st[2] >= s->D && st[2] * eb <= (1ll << 24);
}

// Byte strides of q (heads = Hq) or k (heads = Hkv): the caller's, or the packed layout's.
void byte_strides(const int64_t (&st)[3], const kvcrush_shape* s, int heads, long long& sb, long long& sh,
                  unsigned& rb) {
  const long long eb = (long long)elem_bytes(s);
  if (st[0] == 0 && st[1] == 0 && st[2] == 0) {
    rb = (unsigned)(s->D * eb);
    sh = (long long)s->S * rb;
    sb = (long long)heads * sh;
  } else {
    sb = st[0] * eb;
    sh = st[1] * eb;
    rb = (unsigned)(st[2] * eb);
  }
}

bool shape_ok(const kvcrush_shape* s) {
  if (!s) return false;
  if (s->B < 1 || s->Hq < 1 || s->Hkv < 1 || s->S < 1 || s->D < 1) return false;
  if (s->Hq % s->Hkv != 0) return false;
  if (s->dtype != KVCRUSH_F32 && s->dtype != KVCRUSH_BF16 && s->dtype != KVCRUSH_F16) return false;
  if (s->reduce_groups != 0 && s->reduce_groups != 1) return false;
  if (s->obs_window < 0) return false;
  if (!(s->softmax_scale >= 0.0f) || s->softmax_scale > 1.0e6f) return false;  // also rejects NaN
  return strides_ok(s->q_stride, s) && strides_ok(s->k_stride, s);
}

kvcrush_status scores_entry(const kvcrush_shape* shape, const void* q, const void* k,
                            const float* lse, float* lse_out, float* partial, float2* split_ml,
                            float* scores, bool lse_only, hipStream_t stream) {
  const long long blocks_a = (long long)shape->B * shape->Hq * ((shape->S + 63) / 64);
  if (blocks_a > 0x3FFFFFFFll) return KVCRUSH_ERR_UNSUPPORTED;
  if ((long long)shape->B * shape->Hq > kMaxGridY) return KVCRUSH_ERR_UNSUPPORTED;  // second grid dimension
  ScoreParams p;
  p.q = (const char*)q;
  p.k = (const char*)k;
  byte_strides(shape->q_stride, shape, shape->Hq, p.q_sb, p.q_sh, p.q_rb);
  byte_strides(shape->k_stride, shape, shape->Hkv, p.k_sb, p.k_sh, p.k_rb);
  {
    const long long rb = (long long)shape->D * (long long)elem_bytes(shape), sh = rb * shape->S;
    p.strided = !(p.q_rb == rb && p.k_rb == rb && p.q_sh == sh && p.k_sh == sh && p.q_sb == sh * shape->Hq &&
                  p.k_sb == sh * shape->Hkv);
  }
  p.lse = lse_out;
  p.scores = scores;
  p.partial = partial;
  p.B = shape->B;
  p.Hq = shape->Hq;
  p.Hkv = shape->Hkv;
  p.S = shape->S;
  p.G = shape->Hq / shape->Hkv;
  p.reduce_groups = shape->reduce_groups;
  p.heads_per_wg = 1;
  p.n_blocks = 0;
  p.n_bh = 0;
  p.chunk_tiles = 1;
  p.n_chunks = 1;
  p.n_split = 1;
  p.split_q0 = 0;
  p.split_rows = 0;
  p.split_ml = nullptr;
  p.q_first = first_query(shape);
  p.tile0 = 0;
  p.scale_log2 = (float)(1.4426950408889634 *
                         (shape->softmax_scale != 0.0f ? (double)shape->softmax_scale : 1.0 / sqrt((double)shape->D)));
  if (shape->dtype == KVCRUSH_F16) {
    if (shape->D == 128) return launch_scores<true, 128, true>(p, lse, split_ml, lse_only, stream);
    return launch_scores<true, 64, true>(p, lse, split_ml, lse_only, stream);
  }
  const bool bf16 = shape->dtype == KVCRUSH_BF16;
  if (bf16 && shape->D == 128) return launch_scores<true, 128>(p, lse, split_ml, lse_only, stream);
  if (bf16 && shape->D == 64) return launch_scores<true, 64>(p, lse, split_ml, lse_only, stream);
  if (!bf16 && shape->D == 128) return launch_scores<false, 128>(p, lse, split_ml, lse_only, stream);
  return launch_scores<false, 64>(p, lse, split_ml, lse_only, stream);
}

}  // namespace

extern "C" size_t kvcrush_scores_workspace(const kvcrush_shape* shape) {
  if (!shape_ok(shape)) return 0;
  return lse_bytes(shape) + partial_bytes(shape) + split_bytes(shape);
}

extern "C" size_t kvcrush_row_lse_workspace(const kvcrush_shape* shape) {
  if (!shape_ok(shape)) return 0;
  return split_bytes(shape);
}

extern "C" kvcrush_status kvcrush_scores(const kvcrush_shape* shape, const void* q, const void* k,
                                         const float* lse, float* scores, void* workspace,
                                         size_t workspace_bytes, void* hip_stream) {
  if (!shape_ok(shape)) return KVCRUSH_ERR_INVALID_ARG;
  if (shape->D != 64 && shape->D != 128) return KVCRUSH_ERR_UNSUPPORTED;
  if (!q || !k || !scores) return KVCRUSH_ERR_INVALID_ARG;
  if (!kvc::aligned16(q) || !kvc::aligned16(k) || !kvc::aligned16(scores) || !kvc::aligned16(lse))
    return KVCRUSH_ERR_INVALID_ARG;
  if (!workspace || !kvc::aligned16(workspace) || workspace_bytes < kvcrush_scores_workspace(shape))
    return KVCRUSH_ERR_WORKSPACE;
  float* partial = (float*)((char*)workspace + lse_bytes(shape));
  float2* split_ml =
      split_bytes(shape) ? (float2*)((char*)workspace + lse_bytes(shape) + partial_bytes(shape)) : nullptr;
  return scores_entry(shape, q, k, lse, (float*)workspace, partial, split_ml, scores, false,
                      (hipStream_t)hip_stream);
}

extern "C" kvcrush_status kvcrush_row_lse(const kvcrush_shape* shape, const void* q, const void* k,
                                          float* lse_out, void* workspace, size_t workspace_bytes,
                                          void* hip_stream) {
  if (!shape_ok(shape)) return KVCRUSH_ERR_INVALID_ARG;
  if (shape->D != 64 && shape->D != 128) return KVCRUSH_ERR_UNSUPPORTED;
  if (!q || !k || !lse_out) return KVCRUSH_ERR_INVALID_ARG;
  if (!kvc::aligned16(q) || !kvc::aligned16(k) || !kvc::aligned16(lse_out))
    return KVCRUSH_ERR_INVALID_ARG;
  float2* split_ml = nullptr;
  if (workspace) {
    if (!kvc::aligned16(workspace) || workspace_bytes < split_bytes(shape)) return KVCRUSH_ERR_WORKSPACE;
    if (split_bytes(shape)) split_ml = (float2*)workspace;
  }
  return scores_entry(shape, q, k, nullptr, lse_out, nullptr, split_ml, nullptr, true,
                      (hipStream_t)hip_stream);
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

extern "C" int32_t kvcrush_version(void) { return 120; }

