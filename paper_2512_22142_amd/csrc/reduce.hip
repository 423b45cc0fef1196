// Parameter-server aggregation on the GPU (paper Sec. 3.2: the PS aggregates
// the outputs the devices return): for every output tile the S partial blocks
// are summed in ascending chunk order, ((P0 + P1) + P2) + ..., with plain
// fp32 adds, and the sum is written into C.  Purely HBM-bandwidth bound:
// 4*S bytes read and 4 (or 2) bytes written per output element.
//
// One workgroup handles one reduce item (a run of rows of one tile, ~16K
// elements).  The S blocks of a tile are adjacent in the partial buffer and
// each block is contiguous, so every load of the vector path is a 16-byte
// access into a contiguous stream.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "kernels.h"

namespace cleave {

namespace {

constexpr int kThreads = 256;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Round-to-nearest-even fp32 -> bf16 (NaN stays a quiet NaN).
__device__ __forceinline__ uint32_t to_bf16_bits(float x) {
  uint32_t u = __builtin_bit_cast(uint32_t, x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

template <bool OUT_BF16>
__device__ __forceinline__ void store4(void* C, int64_t off, f32x4 acc) {
  if constexpr (OUT_BF16) {
    u32x2 w;
    w[0] = to_bf16_bits(acc[0]) | (to_bf16_bits(acc[1]) << 16);
    w[1] = to_bf16_bits(acc[2]) | (to_bf16_bits(acc[3]) << 16);
    *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(C) + off) = w;
  } else {
    *reinterpret_cast<f32x4*>(static_cast<float*>(C) + off) = acc;
  }
}

// Vector path for a compile-time split count: all S loads of two output
// float4s are issued before the first add, so every thread keeps 2*S 16-byte
// loads in flight.  The adds stay a left fold in ascending split order.
template <bool OUT_BF16, int S>
__device__ __forceinline__ void reduce_item_fixed(const float* p0, uint64_t block, uint32_t count,
                                                  uint32_t n_len, void* C, int64_t c_base,
                                                  int64_t ldc) {
  constexpr uint32_t kStride = kThreads * 4;
  uint32_t e = threadIdx.x * 4;
  for (; e + kStride < count; e += 2 * kStride) {
    f32x4 a[S], b[S];
#pragma unroll
    for (int s = 0; s < S; ++s) {
      a[s] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p0 + s * block + e));
      b[s] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p0 + s * block + e + kStride));
    }
    f32x4 acc0 = a[0], acc1 = b[0];
#pragma unroll
    for (int s = 1; s < S; ++s) {
      acc0 = acc0 + a[s];
      acc1 = acc1 + b[s];
    }
    const uint32_t r0 = e / n_len, r1 = (e + kStride) / n_len;
    store4<OUT_BF16>(C, c_base + r0 * ldc + (e - r0 * n_len), acc0);
    store4<OUT_BF16>(C, c_base + r1 * ldc + (e + kStride - r1 * n_len), acc1);
  }
  if (e < count) {
    f32x4 a[S];
#pragma unroll
    for (int s = 0; s < S; ++s)
      a[s] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p0 + s * block + e));
    f32x4 acc = a[0];
#pragma unroll
    for (int s = 1; s < S; ++s) acc = acc + a[s];
    const uint32_t r = e / n_len;
    store4<OUT_BF16>(C, c_base + r * ldc + (e - r * n_len), acc);
  }
}

template <bool OUT_BF16, bool VEC>
__global__ __launch_bounds__(kThreads) void reduce_kernel(ReduceArgs args) {
  for (int64_t it = blockIdx.x; it < args.n_items; it += gridDim.x) {
    const ReduceItem item = args.items[it];
    const cleave_task task = args.tasks[item.task];
    const uint32_t n_len = task.n_len;
    const uint32_t S = task.ksplit_cnt;
    const uint64_t block = static_cast<uint64_t>(task.m_len) * n_len;   // elements per partial
    const float* p0 = args.partials + task.partial_off + static_cast<uint64_t>(item.row0) * n_len;
    const uint32_t count = item.rows * n_len;
    const int64_t c_row0 = static_cast<int64_t>(task.m0) + item.row0;
    const int64_t c_base = batch_offset(task.gemm_id, args.batch_inner, args.c_outer, args.c_inner) +
                           c_row0 * args.ldc + task.n0;

    if constexpr (VEC) {
      switch (S) {
        case 1: reduce_item_fixed<OUT_BF16, 1>(p0, block, count, n_len, args.C, c_base, args.ldc); break;
        case 2: reduce_item_fixed<OUT_BF16, 2>(p0, block, count, n_len, args.C, c_base, args.ldc); break;
        case 4: reduce_item_fixed<OUT_BF16, 4>(p0, block, count, n_len, args.C, c_base, args.ldc); break;
        case 8: reduce_item_fixed<OUT_BF16, 8>(p0, block, count, n_len, args.C, c_base, args.ldc); break;
        default:
          for (uint32_t e = threadIdx.x * 4; e < count; e += kThreads * 4) {
            f32x4 acc = *reinterpret_cast<const f32x4*>(p0 + e);
            for (uint32_t s = 1; s < S; ++s)
              acc = acc + *reinterpret_cast<const f32x4*>(p0 + s * block + e);
            const uint32_t r = e / n_len;
            store4<OUT_BF16>(args.C, c_base + r * args.ldc + (e - r * n_len), acc);
          }
      }
    } else {
      for (uint32_t e = threadIdx.x; e < count; e += kThreads) {
        float acc = p0[e];
        for (uint32_t s = 1; s < S; ++s) acc = acc + p0[s * block + e];
        const uint32_t r = e / n_len;
        const int64_t off = c_base + r * args.ldc + (e - r * n_len);
        if constexpr (OUT_BF16) {
          static_cast<uint16_t*>(args.C)[off] = static_cast<uint16_t>(to_bf16_bits(acc));
        } else {
          static_cast<float*>(args.C)[off] = acc;
        }
      }
    }
  }
}

}  // namespace

hipError_t launch_reduce(const ReduceArgs& args, int out_dtype, bool vec, int grid,
                         hipStream_t stream) {
  const dim3 g(grid), b(kThreads);
  if (out_dtype == CLEAVE_BF16) {
    if (vec) hipLaunchKernelGGL((reduce_kernel<true, true>), g, b, 0, stream, args);
    else hipLaunchKernelGGL((reduce_kernel<true, false>), g, b, 0, stream, args);
  } else {
    if (vec) hipLaunchKernelGGL((reduce_kernel<false, true>), g, b, 0, stream, args);
    else hipLaunchKernelGGL((reduce_kernel<false, false>), g, b, 0, stream, args);
  }
  return hipGetLastError();
}

}  // namespace cleave
