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
