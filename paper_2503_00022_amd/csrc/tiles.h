// MFMA tile plumbing shared by the gfx950 kernels that multiply rows of Q and K
// (not part of the ABI).
//
// A tile is kTile rows of one head, D values each.  Tiles travel from global
// memory straight into LDS (global_load_lds_dwordx4, no register staging); rows
// are stored unpadded and the 16-byte chunks of every 256-byte line are
// XOR-swizzled by the line number, which keeps the ds_read_b128 fragment reads
// free of bank conflicts.  The k-index permutation inside an MFMA step is free
// as long as both operands use the same one: lane group g (lane / 32) takes
// chunk  step + g * steps  of a row, i.e. one 16-byte load.
#pragma once
#include "common.h"

namespace kvc {
namespace tiles {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / KVC_WAVE;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;  // finite "no key seen yet": exp2(m_old - m_new) never sees inf - inf

template <bool BF16, int D>
struct Cfg {
  static constexpr int kRowBytes = D * (BF16 ? 2 : 4);
  static constexpr int kSteps = kRowBytes / 32;      // 16-byte fragments per lane and row
  static constexpr int kChunksPerRow = kRowBytes / 16;
  static constexpr int kTile = BF16 ? 64 : 32;       // streamed rows per LDS buffer
  static constexpr int kTileSub = kTile / 32;
  static constexpr int kTileBytes = kTile * kRowBytes;
  static constexpr int kSubBytes = 32 * kRowBytes;
  static constexpr int kLoadsPerWave = kTileBytes / 1024 / kWaves;  // 1 KiB per wave instruction
  static constexpr bool kPipelined = BF16;           // hand-pipelined loop needs two sub-tiles a tile
  static_assert(kTileBytes % (1024 * kWaves) == 0, "tile must split evenly over the waves");
};

// One MFMA "load step": C += A_frag . B_frag^T over this step's k-slice.
// BF16: the operands are 16-bit values (eight per fragment); F16 then says they are IEEE half
// rather than bfloat16 (same layouts and tiling, another matrix instruction).
template <bool BF16, bool F16 = false>
__device__ __forceinline__ void mma_step(f32x16& acc, const u32x4& a, const u32x4& b) {
  if constexpr (BF16 && F16) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                 __builtin_bit_cast(f16x8, b), acc, 0, 0, 0);
  } else if constexpr (BF16) {
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

// Byte offset, inside a tile buffer, of 16-byte chunk `cidx` of row `row`.
template <class C>
__device__ __forceinline__ int lds_chunk_offset(int row, int cidx) {
  const int q = row * C::kChunksPerRow + cidx;
  const int line = q >> 4, pos = q & 15;
  return (line << 8) | ((pos ^ (line & 15)) << 4);
}

// Offset of this lane's step-0 fragment of sub-tile 0; step s is at (off0 ^ (s << 4)),
// sub-tile u adds u * kSubBytes (neither changes the swizzle bits).
template <class C>
__device__ __forceinline__ int lds_frag_offset0(int lane) {
  return lds_chunk_offset<C>(lane & 31, (lane >> 5) * C::kSteps);
}

template <class C>
__device__ __forceinline__ u32x4 lds_frag(const char* buf, int off0, int sub, int step) {
  return *(const u32x4*)(buf + sub * C::kSubBytes + (off0 ^ (step << 4)));
}

// Logical 16-byte chunk (tile row, chunk of the row) that this lane copies with
// its j-th load of a tile (one load per wave instruction; see tile_load_async).
template <class C>
__device__ __forceinline__ void tile_lane_chunk(int wave, int lane, int j, int& row, int& chunk) {
  const int inst = wave + kWaves * j;
  const int p = inst * 64 + lane;  // physical chunk this lane fills
  const int line = p >> 4, pos = (p & 15) ^ (line & 15);
  const int q = line * 16 + pos;   // logical chunk
  row = q / C::kChunksPerRow;
  chunk = q % C::kChunksPerRow;
}

// Per-lane byte offsets of those chunks, relative to a tile's first row, for rows
// that lie `row_bytes` apart in memory (kRowBytes when the rows are packed).
template <class C>
__device__ __forceinline__ void tile_lane_offsets(uint32_t (&rel)[C::kLoadsPerWave], int wave, int lane,
                                                  uint32_t row_bytes = C::kRowBytes) {
#pragma unroll
  for (int j = 0; j < C::kLoadsPerWave; ++j) {
    int row, chunk;
    tile_lane_chunk<C>(wave, lane, j, row, chunk);
    rel[j] = (uint32_t)row * row_bytes + (uint32_t)chunk * 16;
  }
}

// Asynchronous copy of tile rows [row0, row0 + kTile) of one head into an LDS
// buffer: uniform tile address + per-lane offset, no vector address arithmetic.
// Rows past the end of the sequence are clamped to the last row (the callers
// mask or ignore them).  Completion: s_waitcnt vmcnt(0), then a barrier.
template <class C>
__device__ __forceinline__ void tile_load_async(const char* head_base, int row0, int S, char* buf,
                                                const uint32_t (&rel)[C::kLoadsPerWave], int wave, int lane,
                                                uint32_t row_bytes = C::kRowBytes) {
  const char* tile = head_base + (size_t)row0 * row_bytes;
  const int valid = S - row0;  // rows of this tile inside the sequence
#pragma unroll
  for (int j = 0; j < C::kLoadsPerWave; ++j) {
    uint32_t off = rel[j];
    if (valid < C::kTile) {  // ragged last tile (uniform branch)
      int row, chunk;
      tile_lane_chunk<C>(wave, lane, j, row, chunk);
      off = (uint32_t)min(row, valid - 1) * row_bytes + (uint32_t)chunk * 16;
    }
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(tile + off),
                                     (__attribute__((address_space(3))) void*)(buf + (wave + kWaves * j) * 1024),
                                     16, 0, 0);
  }
}

// The same for a tile that lies wholly inside the sequence: no clamping, the
// address is the uniform tile base plus the lane's fixed offset.
template <class C>
__device__ __forceinline__ void tile_load_async_full(const char* head_base, int row0, char* buf,
                                                     const uint32_t (&rel)[C::kLoadsPerWave], int wave,
                                                     uint32_t row_bytes = C::kRowBytes) {
  const char* tile = head_base + (size_t)row0 * row_bytes;
#pragma unroll
  for (int j = 0; j < C::kLoadsPerWave; ++j)
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(tile + rel[j]),
                                     (__attribute__((address_space(3))) void*)(buf + (wave + kWaves * j) * 1024),
                                     16, 0, 0);
}

// The same copy issued as written-out instructions.  The compiler, which cannot tell one LDS
// buffer from another, makes a wave wait for every copy in flight before its next LDS read after
// a copy it knows of: right after the copies were issued, for the whole memory latency.  Copies
// it does not know of cost no such wait; the caller's own wait and barrier at the end of the step
// (which the other form needs as well) are then the only synchronisation, so the buffer must not
// be read before them.  The statement is ordered against barriers and that wait (all of them have
// side effects) but not against LDS reads, which touch other buffers and are free to move across
// it.  M0 holds the wave's LDS destination (one wait state before its use).
// (M0 is a register the compiler reserves and sets itself before each of its own uses; naming it
// as clobbered keeps it from merging such a set across this statement, and draws a warning)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
// `tile` is the tile's first byte and `wave_dst` the LDS byte address of buf + wave * 1024, both
// uniform over the wave (scalar registers): the copy's address is scalar base + the lane's fixed
// 32-bit offset, so a step costs no vector instruction for addresses.
template <class C>
__device__ __forceinline__ void tile_load_async_full_unseen(const char* tile, uint32_t wave_dst,
                                                            const uint32_t (&rel)[C::kLoadsPerWave]) {
#pragma unroll
  for (int j = 0; j < C::kLoadsPerWave; ++j)
    asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(wave_dst), "v"(rel[j]), "s"(tile), "n"(kWaves * j * 1024)
                 : "m0", "scc");
}
// A pointer that is the same in every lane of the wave, moved to scalar registers.
__device__ __forceinline__ const char* wave_uniform(const char* ptr) {
  const uint64_t v = (uint64_t)(uintptr_t)ptr;
  uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  // A memory instruction must not read a scalar register within five wait states of a vector
  // instruction writing it.  The compiler keeps that distance for the instructions it emits
  // itself, but the written-out copies below are opaque to it: keep it here, once.
  asm volatile("s_nop 4" : "+s"(lo), "+s"(hi));
  return (const char*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}
// LDS byte address of a wave's first 1 KiB slot in the buffer at `buf` (uniform over the wave).
__device__ __forceinline__ uint32_t tile_wave_dst(const char* buf, int wave) {
  return __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)(buf + wave * 1024));
}
#pragma clang diagnostic pop

__device__ __forceinline__ void wait_async_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }


// Fragments of 32 stationary rows, straight from global memory to registers
// (zero rows past the end of the sequence).
template <class C>
__device__ __forceinline__ void load_stationary(u32x4 (&frag)[C::kSteps], const char* head_base,
                                                int row0, int S, int lane, uint32_t row_bytes = C::kRowBytes) {
  const int t = row0 + (lane & 31);
#pragma unroll
  for (int s = 0; s < C::kSteps; ++s) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (t < S)
      v = *(const u32x4*)(head_base + (size_t)t * row_bytes + (s + (lane >> 5) * C::kSteps) * 16);
    frag[s] = v;
  }
}

}  // namespace tiles
}  // namespace kvc
