// Sub-GEMM task executor for gfx950 (paper Sec. 4.1: a task multiplies its
// rows of A with its columns of B; here restricted to its chunk of the inner
// dimension, and the fp32 partial block goes to the task's slot in HBM).
//
// This is the staged executor: fp32 inputs, chunk lengths or tile edges the
// bf16 direct-to-LDS path does not take, unaligned operands.  One workgroup
// computes one work item: a 256 x 256 sub-tile (8 wave64 as 2 x 4, a wave owns
// 128 x 64) or a 128 x 128 one (4 waves as 2 x 2, 64 x 64 each) of a task's
// output block over the task's whole chunk [k0, k0 + k_len).  The inner loop
// walks the chunk in ascending steps of 128 bytes of K per row (64 bf16 / 32
// fp32 elements) and, inside a step, in ascending 32-byte sub-steps; the order
// of the MFMA accumulation for an output element therefore depends only on
// the task record, which is what makes a re-issued task bitwise reproducible.
//
// Data path per K step: global -> VGPR (16-byte chunks, issued one step
// ahead) -> LDS (K-contiguous rows, 16 bytes of padding per row so that
// fragment reads are bank-conflict free; operands whose storage is not
// K-contiguous are transposed in registers on the way) -> 16-byte fragment
// reads -> MFMA 32x32x16 bf16 (or 32x32x2 fp32) into fp32 accumulators ->
// stores of the partial block.  The small class is sized so that two
// workgroups share a CU: while one waits at a barrier, refills LDS or drains
// its stores, the other keeps the matrix cores busy.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "plan_internal.h"
#include "kernels.h"
#include "tile_store.h"

namespace cleave {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kChunksPerRow = 8;                    // 128 bytes of K per tile row and step
constexpr int kRowStride = 16 * kChunksPerRow + 16; // LDS bytes per tile row (padded)

// ---------------------------------------------------------------------------
// Operand tile: R rows (an m or n index) x 128 bytes of K, moved global ->
// registers -> LDS by NT threads.  `row_stride` / `k_stride` are element
// strides of the stored matrix along the tile's row index and along K.
// ---------------------------------------------------------------------------
enum LoadMode : int { kVecKContig = 0, kVecTransposed = 1, kScalar = 2 };

template <int EB, int R, int NT, int MODE>
struct OperandTile {
  static constexpr int E = 16 / EB;                 // elements per 16-byte chunk
  static constexpr int NV = R * kChunksPerRow / NT; // 16-byte chunks held per thread
  // Transposed mode: a thread owns KB consecutive k rows x E consecutive tile
  // rows (one 16-byte load per k row) and writes E runs of KB elements.
  static constexpr int KB = (EB == 2) ? (NV < 8 ? NV : 8) : 4;
  static constexpr int kBlocksPerThread = NV / KB;
  static constexpr int KG = kChunksPerRow * E / KB; // k groups per step
  static_assert(NV >= 2 && NV % KB == 0, "unsupported tile / thread count");

  u32x4 v[NV];
  uint32_t off[NV];   // vector modes: byte offset of each 16-byte load from the step base

  // Vector modes: fixes this thread's load offsets for one work item.  Rows
  // beyond r_valid are clamped to the last valid 16-byte run: they only feed
  // output elements that are never stored.
  __device__ __forceinline__ void init(int64_t row_stride, int64_t k_stride, int r_valid, int t) {
    if constexpr (MODE == kVecKContig) {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = t + NT * i;
        const int row = min(c >> 3, r_valid - 1);
        off[i] = static_cast<uint32_t>((row * row_stride + (c & 7) * E) * EB);
      }
    } else if constexpr (MODE == kVecTransposed) {
#pragma unroll
      for (int b = 0; b < kBlocksPerThread; ++b) {
        const int blk = t + NT * b;
        const int kg = (blk >> 3) % KG;
        const int rg = (blk / (8 * KG)) * 8 + (blk & 7);
        const int r = min(rg * E, r_valid - E);
#pragma unroll
        for (int kk = 0; kk < KB; ++kk)
          off[b * KB + kk] = static_cast<uint32_t>(((kg * KB + kk) * k_stride + r) * EB);
      }
    }
  }

  // k index (within the step) of load i, for the tail predicate.
  static __device__ __forceinline__ int k_of(int i, int t) {
    if constexpr (MODE == kVecKContig) {
      return ((t + NT * i) & 7) * E;
    } else {
      const int blk = t + NT * (i / KB);
      return ((blk >> 3) % KG) * KB + (i % KB);
    }
  }

  // base: first element of the tile's row 0 at this step's first k (bytes,
  // wave-uniform).  FULL: the whole step lies inside the chunk; otherwise
  // k_left (>= 1) elements remain and loads beyond them yield zeros.
  template <bool FULL>
  __device__ __forceinline__ void load(const unsigned char* base, int64_t row_stride,
                                       int64_t k_stride, int r_valid, int k_left, int t) {
    if constexpr (MODE != kScalar) {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        if (FULL || k_of(i, t) < k_left) {
          v[i] = *reinterpret_cast<const u32x4*>(base + off[i]);
        } else {
          v[i] = u32x4{0, 0, 0, 0};
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = t + NT * i;
        const int row = c >> 3;
        const int k = (c & 7) * E;
        u32x4 w = {0, 0, 0, 0};
        if (row < r_valid) {
          const unsigned char* p = base + (static_cast<int64_t>(row) * row_stride +
                                           static_cast<int64_t>(k) * k_stride) * EB;
          if constexpr (EB == 4) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (k + e < k_left) w[e] = *reinterpret_cast<const uint32_t*>(p + e * k_stride * 4);
          } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              if (k + e < k_left) {
                const uint32_t h = *reinterpret_cast<const uint16_t*>(p + e * k_stride * 2);
                w[e >> 1] |= h << (16 * (e & 1));
              }
            }
          }
        }
        v[i] = w;
      }
    }
  }

  __device__ __forceinline__ void store(unsigned char* lds, int t) const {
    if constexpr (MODE != kVecTransposed) {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = t + NT * i;
        *reinterpret_cast<u32x4*>(lds + (c >> 3) * kRowStride + (c & 7) * 16) = v[i];
      }
    } else {
#pragma unroll
      for (int b = 0; b < kBlocksPerThread; ++b) {
        const int blk = t + NT * b;
        const int kg = (blk >> 3) % KG;
        const int rg = (blk / (8 * KG)) * 8 + (blk & 7);
        unsigned char* dst = lds + (rg * E) * kRowStride + kg * KB * EB;
        if constexpr (EB == 4) {
          // 4 x 4 transpose of dwords: pure renaming.
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const u32x4 w = {v[b * 4 + 0][j], v[b * 4 + 1][j], v[b * 4 + 2][j], v[b * 4 + 3][j]};
            *reinterpret_cast<u32x4*>(dst + j * kRowStride) = w;
          }
        } else {
          // KB x 8 transpose of 16-bit values: row j of the result collects
          // halfword j of the KB loaded k rows.
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            uint32_t w[KB / 2];
#pragma unroll
            for (int p = 0; p < KB / 2; ++p) {
              const uint32_t lo = v[b * KB + 2 * p][j >> 1];
              const uint32_t hi = v[b * KB + 2 * p + 1][j >> 1];
              w[p] = (j & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
            }
            if constexpr (KB == 8) {
              *reinterpret_cast<u32x4*>(dst + j * kRowStride) = u32x4{w[0], w[1], w[2], w[3]};
            } else if constexpr (KB == 4) {
              *reinterpret_cast<u32x2*>(dst + j * kRowStride) = u32x2{w[0], w[1]};
            } else {
              *reinterpret_cast<uint32_t*>(dst + j * kRowStride) = w[0];
            }
          }
        }
      }
    }
  }
};

// ---------------------------------------------------------------------------
// The kernel.  A TM x TN workgroup tile computed by WM x WN waves; one LDS
// stage (A tile then B tile), refilled from registers between two barriers.
// Two (or more) workgroups are resident per CU, so one workgroup's barriers,
// LDS refills and partial-block stores overlap with the other's MFMAs.
// ---------------------------------------------------------------------------
template <int EB, int TM, int TN, int WM, int WN, int MODE_A, int MODE_B>
__global__ __launch_bounds__(WM* WN * 64, (WM * WN > 4 ? 1 : 2)) void execute_kernel(ExecuteArgs args) {
  constexpr int NT = WM * WN * 64;
  constexpr int E = 16 / EB;
  constexpr int kStepElems = kChunksPerRow * E;
  constexpr int WTM = TM / WM;          // wave tile
  constexpr int WTN = TN / WN;
  constexpr int MB = WTM / 32;          // 32 x 32 MFMA blocks per wave tile
  constexpr int NB = WTN / 32;
  constexpr int kATileBytes = TM * kRowStride;
  constexpr int kSub = kChunksPerRow / 2;   // 32-byte sub-steps per K step

  extern __shared__ __align__(16) unsigned char smem[];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = t >> 6;
  const int wm = wave / WN;
  const int wn = wave % WN;
  const int l32 = lane & 31;
  const int lh = lane >> 5;

  // Element strides of the stored operands along (tile row, K).
  const int64_t a_rs = args.transA ? 1 : args.lda;
  const int64_t a_ks = args.transA ? args.lda : 1;
  const int64_t b_rs = args.transB ? args.ldb : 1;
  const int64_t b_ks = args.transB ? 1 : args.ldb;

  const unsigned char* a_frag = smem + (wm * WTM + l32) * kRowStride + lh * 16;
  const unsigned char* b_frag = smem + kATileBytes + (wn * WTN + l32) * kRowStride + lh * 16;

  for (int64_t it = blockIdx.x; it < args.n_items; it += gridDim.x) {
    const WorkItem item = args.items[it];
    const int m_valid = static_cast<int>(item.m_valid);
    const int n_valid = static_cast<int>(item.n_valid);
    const int64_t m_base = item.m_base;
    const int64_t n_base = item.n_base;
    const int k_len = static_cast<int>(item.k_len);

    const unsigned char* a_ptr =
        static_cast<const unsigned char*>(args.A) +
        (member_offset(args.a_at, args.batch, item.gemm_id) + m_base * a_rs +
         static_cast<int64_t>(item.k0) * a_ks) * EB;
    const unsigned char* b_ptr =
        static_cast<const unsigned char*>(args.B) +
        (member_offset(args.b_at, args.batch, item.gemm_id) + n_base * b_rs +
         static_cast<int64_t>(item.k0) * b_ks) * EB;

    f32x16 acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    OperandTile<EB, TM, NT, MODE_A> ta;
    OperandTile<EB, TN, NT, MODE_B> tb;
    ta.init(a_rs, a_ks, m_valid, t);
    tb.init(b_rs, b_ks, n_valid, t);

    // Global -> registers for step s; full steps take the unpredicated path.
    auto load_step = [&](int s) {
      const int64_t koff = static_cast<int64_t>(s) * kStepElems;
      const int k_left = k_len - static_cast<int>(koff);
      const unsigned char* pa = a_ptr + koff * a_ks * EB;
      const unsigned char* pb = b_ptr + koff * b_ks * EB;
      if (k_left >= kStepElems) {
        ta.template load<true>(pa, a_rs, a_ks, m_valid, k_left, t);
        tb.template load<true>(pb, b_rs, b_ks, n_valid, k_left, t);
      } else {
        ta.template load<false>(pa, a_rs, a_ks, m_valid, k_left, t);
        tb.template load<false>(pb, b_rs, b_ks, n_valid, k_left, t);
      }
    };
    auto store_step = [&]() {
      ta.store(smem, t);
      tb.store(smem + kATileBytes, t);
    };
    u32x4 fa[2][MB], fb[2][NB];
    auto read_frags = [&](int ks, int buf) {
#pragma unroll
      for (int i = 0; i < MB; ++i)
        fa[buf][i] = *reinterpret_cast<const u32x4*>(a_frag + i * 32 * kRowStride + ks * 32);
#pragma unroll
      for (int j = 0; j < NB; ++j)
        fb[buf][j] = *reinterpret_cast<const u32x4*>(b_frag + j * 32 * kRowStride + ks * 32);
    };
    auto mma = [&](int buf) {
#pragma unroll
      for (int i = 0; i < MB; ++i) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          if constexpr (EB == 2) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                __builtin_bit_cast(bf16x8, fa[buf][i]), __builtin_bit_cast(bf16x8, fb[buf][j]),
                acc[i][j], 0, 0, 0);
          } else {
            // (bit-cast the whole chunk first: a bit_cast of a single vector
            // element lvalue is miscompiled into a read of element 0)
            const f32x4 a4 = __builtin_bit_cast(f32x4, fa[buf][i]);
            const f32x4 b4 = __builtin_bit_cast(f32x4, fb[buf][j]);
#pragma unroll
            for (int e = 0; e < 4; ++e)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[e], b4[e], acc[i][j], 0, 0, 0);
          }
        }
      }
    };

    const int steps = (k_len + kStepElems - 1) / kStepElems;
    load_step(0);
    // Every wave has finished reading the previous work item's last tile.
    __syncthreads();
    store_step();
    __syncthreads();

    for (int s = 0; s < steps; ++s) {
      const bool more = s + 1 < steps;
      read_frags(0, 0);
      if (more) load_step(s + 1);
#pragma unroll
      for (int ks = 0; ks < kSub; ++ks) {
        if (ks + 1 < kSub) read_frags(ks + 1, (ks + 1) & 1);
        mma(ks & 1);
        if constexpr (EB == 2) {
          // Issue order inside a sub-step: one fragment read of the next
          // sub-step between consecutive MFMAs of this one.
          if (ks + 1 < kSub) {
#pragma unroll
            for (int x = 0; x < MB + NB; ++x) {
              __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
              __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, MB * NB - (MB + NB), 0);
          }
        }
      }
      if (more) {
        __syncthreads();     // all fragment reads of this step are done
        store_step();
        __syncthreads();     // the next step's tile is visible
      }
    }

    const int row0 = wm * WTM + lh * 4;
    const int col0 = wn * WTN + l32;
    store_tile<MB, NB>(acc, tile_target(args, item), args.C && args.c_bf16, row0, col0, m_valid,
                       n_valid, m_valid == TM && n_valid == TN);
  }
}

template <int EB, int TM, int TN, int WM, int WN, int MODE_A, int MODE_B>
hipError_t launch_one(const ExecuteArgs& args, int grid, hipStream_t stream) {
  constexpr size_t lds = (TM + TN) * kRowStride;
  hipLaunchKernelGGL((execute_kernel<EB, TM, TN, WM, WN, MODE_A, MODE_B>), dim3(grid),
                     dim3(WM * WN * 64), lds, stream, args);
  return hipGetLastError();
}

template <int EB, int TM, int TN, int WM, int WN, int MODE_A, int MODE_B>
hipError_t configure_one() {
  return hipFuncSetAttribute(
      reinterpret_cast<const void*>(execute_kernel<EB, TM, TN, WM, WN, MODE_A, MODE_B>),
      hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>((TM + TN) * kRowStride));
}

template <int EB, int TM, int TN, int WM, int WN>
hipError_t configure_modes() {
  hipError_t e = configure_one<EB, TM, TN, WM, WN, kScalar, kScalar>();
  if (e == hipSuccess) e = configure_one<EB, TM, TN, WM, WN, kVecKContig, kVecKContig>();
  if (e == hipSuccess) e = configure_one<EB, TM, TN, WM, WN, kVecKContig, kVecTransposed>();
  if (e == hipSuccess) e = configure_one<EB, TM, TN, WM, WN, kVecTransposed, kVecKContig>();
  if (e == hipSuccess) e = configure_one<EB, TM, TN, WM, WN, kVecTransposed, kVecTransposed>();
  return e;
}

template <int EB, int TM, int TN, int WM, int WN>
hipError_t launch_modes(const ExecuteArgs& args, bool vec, int grid, hipStream_t stream) {
  if (!vec) return launch_one<EB, TM, TN, WM, WN, kScalar, kScalar>(args, grid, stream);
  const bool a_k = !args.transA;   // A stored M x K: K-contiguous
  const bool b_k = args.transB;    // B stored N x K: K-contiguous
  if (a_k && b_k) return launch_one<EB, TM, TN, WM, WN, kVecKContig, kVecKContig>(args, grid, stream);
  if (a_k && !b_k) return launch_one<EB, TM, TN, WM, WN, kVecKContig, kVecTransposed>(args, grid, stream);
  if (!a_k && b_k) return launch_one<EB, TM, TN, WM, WN, kVecTransposed, kVecKContig>(args, grid, stream);
  return launch_one<EB, TM, TN, WM, WN, kVecTransposed, kVecTransposed>(args, grid, stream);
}

}  // namespace

hipError_t configure_execute_kernels() {
  hipError_t e = configure_modes<2, kLargeTileRows, kLargeTileCols, 2, kLargeTileCols / 64>();
  if (e == hipSuccess) e = configure_modes<2, 128, 128, 2, 2>();
  if (e == hipSuccess) e = configure_modes<4, kLargeTileRows, kLargeTileCols, 2, kLargeTileCols / 64>();
  if (e == hipSuccess) e = configure_modes<4, 128, 128, 2, 2>();
  return e;
}

hipError_t launch_execute(const ExecuteArgs& args, int dtype, int tile_class, bool vec, int grid,
                          hipStream_t stream) {
  if (dtype == CLEAVE_BF16) {
    return tile_class == kTileLarge ? launch_modes<2, kLargeTileRows, kLargeTileCols, 2, kLargeTileCols / 64>(args, vec, grid, stream)
                                    : launch_modes<2, 128, 128, 2, 2>(args, vec, grid, stream);
  }
  return tile_class == kTileLarge ? launch_modes<4, kLargeTileRows, kLargeTileCols, 2, kLargeTileCols / 64>(args, vec, grid, stream)
                                  : launch_modes<4, 128, 128, 2, 2>(args, vec, grid, stream);
}

}  // namespace cleave
