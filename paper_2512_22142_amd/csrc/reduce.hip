// Parameter-server aggregation on the GPU (paper Sec. 3.2: the PS aggregates
// the outputs the devices return): for every output tile the S partial blocks
// are summed in ascending chunk order, ((P0 + P1) + P2) + ..., with plain
// fp32 adds, and the sum is written into C.  Purely HBM-bandwidth bound:
// 4*S bytes read and 4 (or 2) bytes written per output element.  The sum can
// instead feed one of the streaming operators the paper keeps on the PS
// (residual add, Adam update) without being stored first: see the epilogues.
//
// One workgroup handles one reduce item (a run of rows of one tile, ~4K
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

// What happens to an aggregated value.  An epilogue sees the sum of a tile's
// partials (the left fold, unchanged by what follows) for four consecutive
// elements of a row of C, or for one element, at element offset `off` from the
// member's origin; all arrays of one call share the leading dimension ldc.
//
// Store: C = sum, fp32 or bf16 (paper Sec. 3.2: the PS aggregates the outputs).
template <bool OUT_BF16>
struct StoreEpilogue {
  void* C;
  __device__ __forceinline__ const StoreEpilogue& for_member(uint32_t) const { return *this; }
  __device__ __forceinline__ void apply4(int64_t off, f32x4 acc) const {
    if constexpr (OUT_BF16) {
      u32x2 w;
      w[0] = to_bf16_bits(acc[0]) | (to_bf16_bits(acc[1]) << 16);
      w[1] = to_bf16_bits(acc[2]) | (to_bf16_bits(acc[3]) << 16);
      *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(C) + off) = w;
    } else {
      *reinterpret_cast<f32x4*>(static_cast<float*>(C) + off) = acc;
    }
  }
  __device__ __forceinline__ void apply1(int64_t off, float acc) const {
    if constexpr (OUT_BF16) {
      static_cast<uint16_t*>(C)[off] = static_cast<uint16_t>(to_bf16_bits(acc));
    } else {
      static_cast<float*>(C)[off] = acc;
    }
  }
};

// Residual: C = sum + R (a non-GEMM operator kept on the PS, Sec. 4.1), R and
// C of the same element type and layout.
template <bool OUT_BF16>
struct ResidualEpilogue {
  void* C;
  const void* R;
  __device__ __forceinline__ const ResidualEpilogue& for_member(uint32_t) const { return *this; }
  __device__ __forceinline__ void apply4(int64_t off, f32x4 acc) const {
    if constexpr (OUT_BF16) {
      const u32x2 r = *reinterpret_cast<const u32x2*>(static_cast<const uint16_t*>(R) + off);
      acc[0] += __builtin_bit_cast(float, r[0] << 16);
      acc[1] += __builtin_bit_cast(float, r[0] & 0xffff0000u);
      acc[2] += __builtin_bit_cast(float, r[1] << 16);
      acc[3] += __builtin_bit_cast(float, r[1] & 0xffff0000u);
    } else {
      acc = acc + *reinterpret_cast<const f32x4*>(static_cast<const float*>(R) + off);
    }
    StoreEpilogue<OUT_BF16>{C}.apply4(off, acc);
  }
  __device__ __forceinline__ void apply1(int64_t off, float acc) const {
    if constexpr (OUT_BF16) {
      acc += __builtin_bit_cast(float, static_cast<uint32_t>(static_cast<const uint16_t*>(R)[off]) << 16);
    } else {
      acc += static_cast<const float*>(R)[off];
    }
    StoreEpilogue<OUT_BF16>{C}.apply1(off, acc);
  }
};

// Adam on the weight the aggregated values are the gradient of (optimizer
// updates stay on the PS and follow each weight's gradient GEMM, Sec. 4.1 and
// Sec. 6 "Optimizer step accounting and pipelining"): fp32 master weight and
// moments updated in place, bf16 copy of the new weight written when asked
// for.  The gradient itself is never stored.  fp32 arithmetic with correctly
// rounded division and square root; bias corrections arrive as reciprocals
// computed on the host in double.
struct AdamEpilogue {
  float* w;
  float* m;
  float* v;
  uint16_t* w_bf16;   // may be null
  float lr, beta1, beta2, eps, weight_decay, inv_bias1, inv_bias2;
  __device__ __forceinline__ const AdamEpilogue& for_member(uint32_t) const { return *this; }
  __device__ __forceinline__ float update(float g, float w0, float& m_io, float& v_io) const {
    const float m1 = beta1 * m_io + (1.0f - beta1) * g;
    const float v1 = beta2 * v_io + (1.0f - beta2) * (g * g);
    m_io = m1;
    v_io = v1;
    const float m_hat = m1 * inv_bias1;
    const float v_hat = v1 * inv_bias2;
    return w0 - lr * (m_hat / (__builtin_sqrtf(v_hat) + eps) + weight_decay * w0);
  }
  __device__ __forceinline__ void apply4(int64_t off, f32x4 g) const {
    f32x4 w4 = *reinterpret_cast<const f32x4*>(w + off);
    f32x4 m4 = *reinterpret_cast<const f32x4*>(m + off);
    f32x4 v4 = *reinterpret_cast<const f32x4*>(v + off);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float me = m4[e], ve = v4[e];
      w4[e] = update(g[e], w4[e], me, ve);
      m4[e] = me;
      v4[e] = ve;
    }
    *reinterpret_cast<f32x4*>(w + off) = w4;
    *reinterpret_cast<f32x4*>(m + off) = m4;
    *reinterpret_cast<f32x4*>(v + off) = v4;
    if (w_bf16) StoreEpilogue<true>{w_bf16}.apply4(off, w4);
  }
  __device__ __forceinline__ void apply1(int64_t off, float g) const {
    float me = m[off], ve = v[off];
    const float w1 = update(g, w[off], me, ve);
    w[off] = w1;
    m[off] = me;
    v[off] = ve;
    if (w_bf16) w_bf16[off] = static_cast<uint16_t>(to_bf16_bits(w1));
  }
};

// Adam for the weight-gradient GEMMs of one DAG level in one launch: member g of
// the grouped plan updates its own weight, moments and bf16 copy, found through
// one element-offset table per array (from the arrays of member 0).
struct GroupedAdamEpilogue {
  AdamEpilogue first;              // member 0's arrays and the shared hyper-parameters
  int64_t w_at[kMaxGroup], m_at[kMaxGroup], v_at[kMaxGroup], b_at[kMaxGroup];
  __device__ __forceinline__ AdamEpilogue for_member(uint32_t g) const {
    AdamEpilogue e = first;
    e.w += w_at[g];
    e.m += m_at[g];
    e.v += v_at[g];
    if (e.w_bf16) e.w_bf16 += b_at[g];
    return e;
  }
};

// Vector path for a compile-time split count: all S loads of two output
// float4s are issued before the first add, so every thread keeps 2*S 16-byte
// loads in flight.  The adds stay a left fold in ascending split order.
template <int S, typename Epi>
__device__ __forceinline__ void reduce_item_fixed(const float* p0, uint64_t block, uint32_t count,
                                                  uint32_t n_len, const Epi& epi, int64_t c_base,
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
    epi.apply4(c_base + r0 * ldc + (e - r0 * n_len), acc0);
    epi.apply4(c_base + r1 * ldc + (e + kStride - r1 * n_len), acc1);
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
    epi.apply4(c_base + r * ldc + (e - r * n_len), acc);
  }
}

template <typename Epi, bool VEC>
__global__ __launch_bounds__(kThreads) void reduce_kernel(ReduceArgs args, Epi all_members) {
  for (int64_t it = blockIdx.x; it < args.n_items; it += gridDim.x) {
    const ReduceItem item = args.items[it];
    const cleave_task task = args.tasks[item.task];
    const auto epi = all_members.for_member(task.gemm_id);
    const uint32_t n_len = task.n_len;
    const uint32_t S = task.ksplit_cnt;
    const uint64_t block = static_cast<uint64_t>(task.m_len) * n_len;   // elements per partial
    const float* p0 = args.partials + task.partial_off + static_cast<uint64_t>(item.row0) * n_len;
    const uint32_t count = item.rows * n_len;
    const int64_t c_row0 = static_cast<int64_t>(task.m0) + item.row0;
    const int64_t c_base = member_offset(args.c_at, args.batch, task.gemm_id) +
                           c_row0 * args.ldc + task.n0;

    if constexpr (VEC) {
      switch (S) {
        case 1: reduce_item_fixed<1>(p0, block, count, n_len, epi, c_base, args.ldc); break;
        case 2: reduce_item_fixed<2>(p0, block, count, n_len, epi, c_base, args.ldc); break;
        case 4: reduce_item_fixed<4>(p0, block, count, n_len, epi, c_base, args.ldc); break;
        case 8: reduce_item_fixed<8>(p0, block, count, n_len, epi, c_base, args.ldc); break;
        default:
          for (uint32_t e = threadIdx.x * 4; e < count; e += kThreads * 4) {
            f32x4 acc = *reinterpret_cast<const f32x4*>(p0 + e);
            for (uint32_t s = 1; s < S; ++s)
              acc = acc + *reinterpret_cast<const f32x4*>(p0 + s * block + e);
            const uint32_t r = e / n_len;
            epi.apply4(c_base + r * args.ldc + (e - r * n_len), acc);
          }
      }
    } else {
      for (uint32_t e = threadIdx.x; e < count; e += kThreads) {
        float acc = p0[e];
        for (uint32_t s = 1; s < S; ++s) acc = acc + p0[s * block + e];
        const uint32_t r = e / n_len;
        epi.apply1(c_base + r * args.ldc + (e - r * n_len), acc);
      }
    }
  }
}

template <typename Epi>
hipError_t launch_with(const ReduceArgs& args, const Epi& epi, bool vec, int grid, hipStream_t stream) {
  const dim3 g(grid), b(kThreads);
  if (vec) hipLaunchKernelGGL((reduce_kernel<Epi, true>), g, b, 0, stream, args, epi);
  else hipLaunchKernelGGL((reduce_kernel<Epi, false>), g, b, 0, stream, args, epi);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_reduce(const ReduceArgs& args, int out_dtype, bool vec, int grid,
                         hipStream_t stream) {
  if (out_dtype == CLEAVE_BF16) return launch_with(args, StoreEpilogue<true>{args.C}, vec, grid, stream);
  return launch_with(args, StoreEpilogue<false>{args.C}, vec, grid, stream);
}

hipError_t launch_reduce_residual(const ReduceArgs& args, const void* R, int out_dtype, bool vec,
                                  int grid, hipStream_t stream) {
  if (out_dtype == CLEAVE_BF16)
    return launch_with(args, ResidualEpilogue<true>{args.C, R}, vec, grid, stream);
  return launch_with(args, ResidualEpilogue<false>{args.C, R}, vec, grid, stream);
}

hipError_t launch_reduce_adam(const ReduceArgs& args, const AdamArgs& h, bool vec, int grid,
                              hipStream_t stream) {
  const AdamEpilogue epi{h.w, h.m, h.v, h.w_bf16, h.lr, h.beta1, h.beta2, h.eps,
                         h.weight_decay, h.inv_bias1, h.inv_bias2};
  return launch_with(args, epi, vec, grid, stream);
}

hipError_t launch_reduce_adam_grouped(const ReduceArgs& args, const AdamArgs& h, const AdamGroupOffsets& at,
                                      bool vec, int grid, hipStream_t stream) {
  GroupedAdamEpilogue epi{};
  epi.first = AdamEpilogue{h.w, h.m, h.v, h.w_bf16, h.lr, h.beta1, h.beta2, h.eps,
                           h.weight_decay, h.inv_bias1, h.inv_bias2};
  for (int g = 0; g < kMaxGroup; ++g) {
    epi.w_at[g] = at.w[g];
    epi.m_at[g] = at.m[g];
    epi.v_at[g] = at.v[g];
    epi.b_at[g] = at.w_bf16[g];
  }
  return launch_with(args, epi, vec, grid, stream);
}

}  // namespace cleave
