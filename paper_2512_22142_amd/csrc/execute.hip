// Sub-GEMM task executor for gfx950 (paper Sec. 4.1: a task multiplies its
// rows of A with its columns of B; here restricted to its chunk of the inner
// dimension, and the fp32 partial block goes to the task's slot in HBM).
//
// One workgroup (256 threads = 4 wave64, arranged 2 x 2) computes one work
// item: an EDGE x EDGE sub-tile of a task's output block over the task's whole
// chunk [k0, k0 + k_len).  The inner loop walks the chunk in ascending steps
// of 128 bytes of K per row (64 bf16 / 32 fp32 elements); the order of the
// MFMA accumulation for an output element therefore depends only on the task
// record, which is what makes a re-issued task bitwise reproducible.
//
// Data path per K step: global -> VGPR (16-byte chunks, next step prefetched
// while the current one is multiplied) -> LDS (K-contiguous rows, 16 bytes of
// padding per row so that fragment reads are bank-conflict free; operands
// whose storage is not K-contiguous are transposed in registers on the way)
// -> 16-byte fragment reads -> MFMA 32x32x16 bf16 (or 32x32x2 fp32) into fp32
// accumulators -> guarded stores of the partial block.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "plan_internal.h"
#include "kernels.h"

namespace cleave {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kChunksPerRow = 8;                    // 128 bytes of K per tile row and step
constexpr int kRowStride = 16 * kChunksPerRow + 16; // LDS bytes per tile row (padded)

// ---------------------------------------------------------------------------
// Operand tile: R rows (an m or n index) x 128 bytes of K, moved global ->
// registers -> LDS.  `row_stride` / `k_stride` are element strides of the
// stored matrix along the tile's row index and along K.
// ---------------------------------------------------------------------------
enum LoadMode : int { kVecKContig = 0, kVecTransposed = 1, kScalar = 2 };

template <int EB, int R, int MODE>
struct OperandTile {
  static constexpr int E = 16 / EB;                 // elements per 16-byte chunk
  static constexpr int kStepElems = kChunksPerRow * E;
  static constexpr int NV = R / 32;                 // chunks held per thread
  static constexpr int kBlocks = kChunksPerRow * (R / E);   // E x E blocks (transposed mode)
  static constexpr int kBlocksPerThread = (kBlocks + kThreads - 1) / kThreads;
  static constexpr int NREG = MODE == kVecTransposed ? kBlocksPerThread * E : NV;

  u32x4 v[NREG];

  // base: first element of the tile's row 0 at the chunk start k0 (bytes).
  // r_valid: rows of the tile that exist; k_left: elements of K that remain
  // from this step's start (>= 1).
  __device__ __forceinline__ void load(const unsigned char* base, int64_t row_stride,
                                       int64_t k_stride, int r_valid, int k_left, int t) {
    if constexpr (MODE == kVecKContig) {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = t + kThreads * i;
        const int row = min(c >> 3, r_valid - 1);
        const int k = (c & 7) * E;
        const unsigned char* p = base + (static_cast<int64_t>(row) * row_stride + k) * EB;
        v[i] = (k < k_left) ? *reinterpret_cast<const u32x4*>(p) : u32x4{0, 0, 0, 0};
      }
    } else if constexpr (MODE == kVecTransposed) {
#pragma unroll
      for (int b = 0; b < kBlocksPerThread; ++b) {
        const int blk = t + kThreads * b;
        const int kg = blk & 7;
        const int rg = blk >> 3;
        const int r = min(rg * E, r_valid - E);
#pragma unroll
        for (int kk = 0; kk < E; ++kk) {
          const int k = kg * E + kk;
          const unsigned char* p = base + (static_cast<int64_t>(k) * k_stride + r) * EB;
          const bool ok = (kBlocks >= kThreads || blk < kBlocks) && k < k_left;
          v[b * E + kk] = ok ? *reinterpret_cast<const u32x4*>(p) : u32x4{0, 0, 0, 0};
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = t + kThreads * i;
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
        const int c = t + kThreads * i;
        *reinterpret_cast<u32x4*>(lds + (c >> 3) * kRowStride + (c & 7) * 16) = v[i];
      }
    } else {
#pragma unroll
      for (int b = 0; b < kBlocksPerThread; ++b) {
        const int blk = t + kThreads * b;
        if (kBlocks < kThreads && blk >= kBlocks) continue;
        const int kg = blk & 7;
        const int rg = blk >> 3;
        unsigned char* dst = lds + (rg * E) * kRowStride + kg * 16;
        if constexpr (EB == 4) {
          // 4 x 4 transpose of dwords: pure renaming.
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const u32x4 w = {v[b * 4 + 0][j], v[b * 4 + 1][j], v[b * 4 + 2][j], v[b * 4 + 3][j]};
            *reinterpret_cast<u32x4*>(dst + j * kRowStride) = w;
          }
        } else {
          // 8 x 8 transpose of 16-bit values: row j of the result collects
          // halfword j of the eight loaded k rows.
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            u32x4 w;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
              const uint32_t lo = v[b * 8 + 2 * p][j >> 1];
              const uint32_t hi = v[b * 8 + 2 * p + 1][j >> 1];
              w[p] = (j & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
            }
            *reinterpret_cast<u32x4*>(dst + j * kRowStride) = w;
          }
        }
      }
    }
  }
};

// ---------------------------------------------------------------------------
// The kernel.
// ---------------------------------------------------------------------------
template <int EB, int EDGE, int MODE_A, int MODE_B>
__global__ __launch_bounds__(kThreads) void execute_kernel(ExecuteArgs args) {
  constexpr int E = 16 / EB;
  constexpr int kStepElems = kChunksPerRow * E;
  constexpr int WT = EDGE / 2;          // wave tile edge
  constexpr int NBLK = WT / 32;         // 32 x 32 MFMA blocks per wave tile edge
  constexpr int kTileBytes = EDGE * kRowStride;
  constexpr int kStageBytes = 2 * kTileBytes;

  extern __shared__ __align__(16) unsigned char smem[];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = t >> 6;
  const int wm = wave >> 1;
  const int wn = wave & 1;
  const int l32 = lane & 31;
  const int lh = lane >> 5;

  // Element strides of the stored operands along (tile row, K).
  const int64_t a_rs = args.transA ? 1 : args.lda;
  const int64_t a_ks = args.transA ? args.lda : 1;
  const int64_t b_rs = args.transB ? args.ldb : 1;
  const int64_t b_ks = args.transB ? 1 : args.ldb;

  for (int64_t it = blockIdx.x; it < args.n_items; it += gridDim.x) {
    const WorkItem item = args.items[it];
    const cleave_task task = args.tasks[item.task];
    const uint32_t sub_cols = (task.n_len + EDGE - 1) / EDGE;
    const uint32_t sub_m = item.sub / sub_cols;
    const uint32_t sub_n = item.sub - sub_m * sub_cols;
    const int m_valid = min(static_cast<int>(task.m_len - sub_m * EDGE), EDGE);
    const int n_valid = min(static_cast<int>(task.n_len - sub_n * EDGE), EDGE);
    const int64_t m_base = static_cast<int64_t>(task.m0) + static_cast<int64_t>(sub_m) * EDGE;
    const int64_t n_base = static_cast<int64_t>(task.n0) + static_cast<int64_t>(sub_n) * EDGE;
    const int k_len = static_cast<int>(task.k_len);

    const unsigned char* a_ptr = static_cast<const unsigned char*>(args.A) +
                                 (m_base * a_rs + static_cast<int64_t>(task.k0) * a_ks) * EB;
    const unsigned char* b_ptr = static_cast<const unsigned char*>(args.B) +
                                 (n_base * b_rs + static_cast<int64_t>(task.k0) * b_ks) * EB;

    f32x16 acc[NBLK][NBLK];
#pragma unroll
    for (int i = 0; i < NBLK; ++i)
#pragma unroll
      for (int j = 0; j < NBLK; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    OperandTile<EB, EDGE, MODE_A> ta;
    OperandTile<EB, EDGE, MODE_B> tb;

    const int steps = (k_len + kStepElems - 1) / kStepElems;
    ta.load(a_ptr, a_rs, a_ks, m_valid, k_len, t);
    tb.load(b_ptr, b_rs, b_ks, n_valid, k_len, t);
    ta.store(smem, t);
    tb.store(smem + kTileBytes, t);
    __syncthreads();

    for (int s = 0; s < steps; ++s) {
      unsigned char* cur = smem + (s & 1) * kStageBytes;
      unsigned char* nxt = smem + ((s + 1) & 1) * kStageBytes;
      const bool more = s + 1 < steps;
      if (more) {
        const int64_t koff = static_cast<int64_t>(s + 1) * kStepElems;
        const int k_left = k_len - static_cast<int>(koff);
        ta.load(a_ptr + koff * a_ks * EB, a_rs, a_ks, m_valid, k_left, t);
        tb.load(b_ptr + koff * b_ks * EB, b_rs, b_ks, n_valid, k_left, t);
      }

      const unsigned char* a_frag = cur + (wm * WT + l32) * kRowStride + lh * 16;
      const unsigned char* b_frag = cur + kTileBytes + (wn * WT + l32) * kRowStride + lh * 16;
#pragma unroll
      for (int ks = 0; ks < kChunksPerRow / 2; ++ks) {
        u32x4 af[NBLK], bf[NBLK];
#pragma unroll
        for (int i = 0; i < NBLK; ++i)
          af[i] = *reinterpret_cast<const u32x4*>(a_frag + i * 32 * kRowStride + ks * 32);
#pragma unroll
        for (int j = 0; j < NBLK; ++j)
          bf[j] = *reinterpret_cast<const u32x4*>(b_frag + j * 32 * kRowStride + ks * 32);
#pragma unroll
        for (int i = 0; i < NBLK; ++i) {
#pragma unroll
          for (int j = 0; j < NBLK; ++j) {
            if constexpr (EB == 2) {
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                  __builtin_bit_cast(bf16x8, af[i]), __builtin_bit_cast(bf16x8, bf[j]), acc[i][j],
                  0, 0, 0);
            } else {
              // (bit-cast the whole chunk first: a bit_cast of a single vector
              // element lvalue is miscompiled into a read of element 0)
              const f32x4 a4 = __builtin_bit_cast(f32x4, af[i]);
              const f32x4 b4 = __builtin_bit_cast(f32x4, bf[j]);
#pragma unroll
              for (int e = 0; e < 4; ++e)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[e], b4[e], acc[i][j], 0, 0, 0);
            }
          }
        }
      }

      if (more) {
        ta.store(nxt, t);
        tb.store(nxt + kTileBytes, t);
      }
      __syncthreads();
    }

    // Partial block: row-major m_len x n_len at partial_off.  A 32 x 32 MFMA
    // block leaves lane l with column l % 32 and rows 8*q + 4*(l / 32) + r.
    float* out = args.partials + task.partial_off;
    const int64_t ldp = task.n_len;
#pragma unroll
    for (int i = 0; i < NBLK; ++i) {
#pragma unroll
      for (int j = 0; j < NBLK; ++j) {
        const int col = wn * WT + j * 32 + l32;
        if (col >= n_valid) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int row = wm * WT + i * 32 + q * 8 + lh * 4 + r;
            if (row < m_valid)
              out[(static_cast<int64_t>(sub_m) * EDGE + row) * ldp + sub_n * EDGE + col] =
                  acc[i][j][q * 4 + r];
          }
        }
      }
    }
  }
}

template <int EB, int EDGE, int MODE_A, int MODE_B>
hipError_t launch_one(const ExecuteArgs& args, int grid, hipStream_t stream) {
  constexpr size_t lds = 2 * 2 * EDGE * kRowStride;
  auto kern = execute_kernel<EB, EDGE, MODE_A, MODE_B>;
  static thread_local int configured_device = -1;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (configured_device != dev) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (e != hipSuccess) return e;
    configured_device = dev;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, stream, args);
  return hipGetLastError();
}

template <int EB, int EDGE>
hipError_t launch_modes(const ExecuteArgs& args, bool vec, int grid, hipStream_t stream) {
  if (!vec) return launch_one<EB, EDGE, kScalar, kScalar>(args, grid, stream);
  const bool a_k = !args.transA;   // A stored M x K: K-contiguous
  const bool b_k = args.transB;    // B stored N x K: K-contiguous
  if (a_k && b_k) return launch_one<EB, EDGE, kVecKContig, kVecKContig>(args, grid, stream);
  if (a_k && !b_k) return launch_one<EB, EDGE, kVecKContig, kVecTransposed>(args, grid, stream);
  if (!a_k && b_k) return launch_one<EB, EDGE, kVecTransposed, kVecKContig>(args, grid, stream);
  return launch_one<EB, EDGE, kVecTransposed, kVecTransposed>(args, grid, stream);
}

}  // namespace

hipError_t launch_execute(const ExecuteArgs& args, int dtype, int tile_class, bool vec, int grid,
                          hipStream_t stream) {
  if (dtype == CLEAVE_BF16) {
    return tile_class == kTileLarge ? launch_modes<2, 256>(args, vec, grid, stream)
                                    : launch_modes<2, 128>(args, vec, grid, stream);
  }
  return tile_class == kTileLarge ? launch_modes<4, 256>(args, vec, grid, stream)
                                  : launch_modes<4, 128>(args, vec, grid, stream);
}

}  // namespace cleave
