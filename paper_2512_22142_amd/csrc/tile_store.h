// Where a work item's accumulators go, and the stores that put them there;
// shared by the two execute kernels.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "kernels.h"

namespace cleave {

typedef float tile_f32x16 __attribute__((ext_vector_type(16)));

// Destination of one sub-tile: element (0, 0) of the sub-tile and the row
// stride in elements (the element type is a property of the launch:
// ExecuteArgs::c_bf16).
struct TileTarget {
  unsigned char* base;
  int64_t ld;
};

// Partial mode (args.C == nullptr): the benchmark's fp32 block, row-major
// m_len x n_len at partial_off (paper Sec. 4.1: a device returns its
// alpha x beta block).  Assemble mode: the block's place in the output matrix
// itself (Sec. 3.2: the PS assembles the returned blocks) -- only meaningful
// for tasks that cover the whole inner dimension.
__device__ __forceinline__ TileTarget tile_target(const ExecuteArgs& args, const WorkItem& w) {
  TileTarget t;
  if (args.C == nullptr) {
    t.ld = w.out_ld;
    t.base = reinterpret_cast<unsigned char*>(args.partials + w.out_off);
  } else {
    t.ld = args.ldc;
    const int64_t off = member_offset(args.c_at, args.batch, w.gemm_id) +
                        static_cast<int64_t>(w.m_base) * t.ld + w.n_base;
    t.base = static_cast<unsigned char*>(args.C) + off * (args.c_bf16 ? 2 : 4);
  }
  return t;
}

// Round-to-nearest-even fp32 -> bf16 (NaN stays a quiet NaN).
__device__ __forceinline__ uint16_t tile_to_bf16(float x) {
  uint32_t u = __builtin_bit_cast(uint32_t, x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

// Stores a wave's MB x NB grid of 32 x 32 MFMA accumulator blocks.  A block
// leaves lane l with column l % 32 and rows 8*q + 4*(l / 32) + r, so half a
// wave writes one aligned run of 32 elements per store.  row0 / col0: this
// lane's first row and column inside the sub-tile; one per-thread base pointer
// plus wave-uniform row offsets keeps the stores free of address arithmetic.
// `interior`: the sub-tile is full, no bounds checks.  Plain stores:
// non-temporal ones make execute ~1 % faster but the reducer that follows
// ~10 % slower.
template <int MB, int NB, typename T, typename Cvt>
__device__ __forceinline__ void store_blocks(const tile_f32x16 (&acc)[MB][NB], T* tp, int64_t ld,
                                             int row0, int col0, int m_valid, int n_valid,
                                             bool interior, Cvt cvt) {
  if (interior) {
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          T* p = tp + static_cast<int64_t>(i * 32 + q * 8 + r) * ld;
#pragma unroll
          for (int j = 0; j < NB; ++j) p[j * 32] = cvt(acc[i][j][q * 4 + r]);
        }
  } else {
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int rr = i * 32 + q * 8 + r;
          T* p = tp + static_cast<int64_t>(rr) * ld;
#pragma unroll
          for (int j = 0; j < NB; ++j)
            if (row0 + rr < m_valid && col0 + j * 32 < n_valid) p[j * 32] = cvt(acc[i][j][q * 4 + r]);
        }
  }
}

// Block rows [I0, I1) of a full sub-tile (no bounds checks), same order and
// addresses as store_blocks: lets a caller put other work between two parts
// of a sub-tile's stores.
template <int MB, int NB, int I0, int I1, typename T, typename Cvt>
__device__ __forceinline__ void store_block_rows(const tile_f32x16 (&acc)[MB][NB], T* tp, int64_t ld,
                                                 Cvt cvt) {
#pragma unroll
  for (int i = I0; i < I1; ++i)
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        T* p = tp + static_cast<int64_t>(i * 32 + q * 8 + r) * ld;
#pragma unroll
        for (int j = 0; j < NB; ++j) p[j * 32] = cvt(acc[i][j][q * 4 + r]);
      }
}

template <int MB, int NB, int I0, int I1>
__device__ __forceinline__ void store_tile_rows(const tile_f32x16 (&acc)[MB][NB], const TileTarget& t,
                                                bool bf16, int row0, int col0) {
  if (!bf16) {
    float* tp = reinterpret_cast<float*>(t.base) + row0 * t.ld + col0;
    store_block_rows<MB, NB, I0, I1>(acc, tp, t.ld, [](float x) { return x; });
  } else {
    uint16_t* tp = reinterpret_cast<uint16_t*>(t.base) + row0 * t.ld + col0;
    store_block_rows<MB, NB, I0, I1>(acc, tp, t.ld, [](float x) { return tile_to_bf16(x); });
  }
}

// Number of store instructions a lane issues for a full sub-tile.
template <int MB, int NB>
__device__ __forceinline__ constexpr int full_tile_stores() {
  return MB * NB * 16;
}

// Block rows [I0, I1) of a full sub-tile, each 32 x 32 block turned through a
// 4 KB row-major image in LDS that belongs to this wave alone (`image`), so
// that a lane leaves with four consecutive columns of one row: a store
// instruction then writes eight whole 128-byte lines (fp32) instead of 64
// dwords in two rows -- a quarter of the store instructions and half the
// address-unit cycles of store_block_rows.  The values and their addresses are
// the same.  wave_row0 / wave_col0: first row and column of the wave's part
// of the sub-tile.  The target must allow 16-byte (fp32) or 8-byte (bf16)
// stores at every fourth column.  LDS executes a wave's accesses in issue
// order, and the compiler is kept from reordering them by the asm statements;
// no other wave touches the image, so no barrier is involved.
constexpr int kBlockImageBytes = 32 * 32 * 4;
template <int NB>
__device__ __forceinline__ constexpr int staged_stores_per_block_row() {
  return NB * 4;
}

template <int MB, int NB, int I0, int I1>
__device__ __forceinline__ void store_tile_rows_staged(const tile_f32x16 (&acc)[MB][NB],
                                                       const TileTarget& t, bool bf16,
                                                       unsigned char* image, int wave_row0,
                                                       int wave_col0, int lane) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  float* wr = reinterpret_cast<float*>(image) + (4 * (lane >> 5)) * 32 + (lane & 31);
  const f32x4* rd = reinterpret_cast<const f32x4*>(image) + lane;   // row lane / 8 (+ 8 k), columns 4 (lane % 8) ..
  const int64_t at = static_cast<int64_t>(wave_row0 + (lane >> 3)) * t.ld + wave_col0 + (lane & 7) * 4;
  float* gp32 = reinterpret_cast<float*>(t.base) + at;
  uint16_t* gp16 = reinterpret_cast<uint16_t*>(t.base) + at;
#pragma unroll
  for (int i = I0; i < I1; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      asm volatile("" ::: "memory");
#pragma unroll
      for (int r = 0; r < 16; ++r) wr[((r >> 2) * 8 + (r & 3)) * 32] = acc[i][j][r];
      asm volatile("" ::: "memory");
      f32x4 v[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) v[k] = rd[64 * k];
      asm volatile("" ::: "memory");
      const int64_t block_at = static_cast<int64_t>(i * 32) * t.ld + j * 32;
      if (!bf16) {
#pragma unroll
        for (int k = 0; k < 4; ++k) *reinterpret_cast<f32x4*>(gp32 + block_at + 8 * k * t.ld) = v[k];
      } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          u32x2 w;
          w[0] = tile_to_bf16(v[k][0]) | (static_cast<uint32_t>(tile_to_bf16(v[k][1])) << 16);
          w[1] = tile_to_bf16(v[k][2]) | (static_cast<uint32_t>(tile_to_bf16(v[k][3])) << 16);
          *reinterpret_cast<u32x2*>(gp16 + block_at + 8 * k * t.ld) = w;
        }
      }
    }
}

template <int MB, int NB>
__device__ __forceinline__ void store_tile(const tile_f32x16 (&acc)[MB][NB], const TileTarget& t,
                                           bool bf16, int row0, int col0, int m_valid,
                                           int n_valid, bool interior) {
  if (!bf16) {
    float* tp = reinterpret_cast<float*>(t.base) + row0 * t.ld + col0;
    store_blocks<MB, NB>(acc, tp, t.ld, row0, col0, m_valid, n_valid, interior,
                         [](float x) { return x; });
  } else {
    uint16_t* tp = reinterpret_cast<uint16_t*>(t.base) + row0 * t.ld + col0;
    store_blocks<MB, NB>(acc, tp, t.ld, row0, col0, m_valid, n_valid, interior,
                         [](float x) { return tile_to_bf16(x); });
  }
}

}  // namespace cleave
