// Returned-block check on the GPU (paper Sec. 6, "Robustness to poisoning
// attacks"): the aggregator dispatched the rows of A and the columns of B of a
// task and received the block P; for probe vectors r, s it accepts P when
//     r^T P s  =  (A_blk^T r)^T (B_blk s)
// up to rounding.  Everything here is matrix-vector work, bound by HBM
// bandwidth: every partial block is read once, the operands once per distinct
// row / column segment of the tiling.  All sums are carried in fp64 (the
// vector fp64 rate is far above what the memory system feeds), each in a fixed
// order, so the results are reproducible and exact for integer-valued inputs.
//
// Three kernels:
//   project_*   U[seg][k] = sum_i op(A)[i][k] r[i] over a row segment (and the
//               same with absolute values), V[seg][k] likewise for op(B), s;
//   bilinear    per run of rows of a partial block: sum_i r_i sum_j P_ij s_j;
//   verdict     per task: lhs from its item sums, rhs = sum_k U_k V_k and
//               scale = sum_k |U|_k |V|_k over the task's chunk, and the
//               decision |lhs - rhs| <= tol * scale.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "kernels.h"

namespace cleave {

namespace {

constexpr int kThreads = 256;
constexpr int kMaxGridY = 65535;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ double bf16_bits_to_double(uint32_t bits16) {
  return static_cast<double>(__builtin_bit_cast(float, bits16 << 16));
}

// VEC consecutive stored elements starting at element index `idx` of `src`, widened exactly.
template <int EB, int VEC>
__device__ __forceinline__ void load_elems(const void* src, int64_t idx, double (&x)[VEC]) {
  if constexpr (EB == 2 && VEC == 8) {
    const u32x4 v = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(src) + idx);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      x[2 * e] = bf16_bits_to_double(v[e] & 0xffffu);
      x[2 * e + 1] = bf16_bits_to_double(v[e] >> 16);
    }
  } else if constexpr (EB == 4 && VEC == 4) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(static_cast<const float*>(src) + idx);
#pragma unroll
    for (int e = 0; e < 4; ++e) x[e] = static_cast<double>(v[e]);
  } else {
    static_assert(VEC == 1, "vector widths: 8 bf16, 4 fp32, or 1");
    if constexpr (EB == 2) {
      x[0] = bf16_bits_to_double(static_cast<const uint16_t*>(src)[idx]);
    } else {
      x[0] = static_cast<double>(static_cast<const float*>(src)[idx]);
    }
  }
}

// Sum over the 64 lanes of a wave, same tree on every call.
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}

// The summed index strides through memory (x(i, k) = src[i * ld + k]); a thread
// owns VEC consecutive k and every SL-th row of the segment, the SL row slices
// are then added in ascending order.
template <int EB, int VEC>
__global__ __launch_bounds__(kThreads) void project_strided_kernel(ProjectArgs a) {
  constexpr int KT = VEC == 1 ? 64 : 8;      // threads along k
  constexpr int SL = kThreads / KT;          // row slices
  constexpr int KW = KT * VEC;               // k per workgroup
  __shared__ double red[2][SL][KW];

  const int t = threadIdx.x;
  const int slice = t / KT;
  const int64_t k = static_cast<int64_t>(blockIdx.x) * KW + (t % KT) * VEC;
  // the grid's second dimension is capped; a workgroup may own several segments
  for (int si = blockIdx.y; si < a.n_segs; si += gridDim.y) {
  const Segment seg = a.segs[si];
  double acc[VEC], acc_abs[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = acc_abs[e] = 0.0;
  if (k < a.K) {
#pragma unroll 4
    for (uint32_t i = slice; i < seg.len; i += SL) {
      const int64_t row = static_cast<int64_t>(seg.start) + i;
      const double w = static_cast<double>(a.w[row]);
      double x[VEC];
      load_elems<EB, VEC>(a.src, row * a.ld + k, x);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        acc[e] = fma(x[e], w, acc[e]);
        acc_abs[e] = fma(fabs(x[e]), fabs(w), acc_abs[e]);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    red[0][slice][(t % KT) * VEC + e] = acc[e];
    red[1][slice][(t % KT) * VEC + e] = acc_abs[e];
  }
  __syncthreads();
  if (t < KW) {
    const int64_t ko = static_cast<int64_t>(blockIdx.x) * KW + t;
    if (ko < a.K) {
      double s0 = 0.0, s1 = 0.0;
#pragma unroll
      for (int sl = 0; sl < SL; ++sl) {
        s0 += red[0][sl][t];
        s1 += red[1][sl][t];
      }
      a.out[static_cast<int64_t>(si) * a.K + ko] = s0;
      a.out_abs[static_cast<int64_t>(si) * a.K + ko] = s1;
    }
  }
  __syncthreads();   // red is reused by the next segment
  }
}

// The summed index is contiguous (x(i, k) = src[k * ld + i]): one wave per
// (segment, k), lanes stride over the segment, fixed reduction tree.
template <int EB, int VEC>
__global__ __launch_bounds__(kThreads) void project_rows_kernel(ProjectArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t k = static_cast<int64_t>(blockIdx.x) * (kThreads / 64) + (threadIdx.x >> 6);
  if (k >= a.K) return;   // whole waves leave together; no barrier below
  for (int si = blockIdx.y; si < a.n_segs; si += gridDim.y) {
  const Segment seg = a.segs[si];
  const int64_t base = k * a.ld + seg.start;
  double acc = 0.0, acc_abs = 0.0;
  for (uint32_t i = lane * VEC; i < seg.len; i += 64 * VEC) {
    double x[VEC];
    load_elems<EB, VEC>(a.src, base + i, x);
    float w[VEC];
    if constexpr (VEC == 8) {
      const f32x4 w0 = *reinterpret_cast<const f32x4*>(a.w + seg.start + i);
      const f32x4 w1 = *reinterpret_cast<const f32x4*>(a.w + seg.start + i + 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        w[e] = w0[e];
        w[4 + e] = w1[e];
      }
    } else if constexpr (VEC == 4) {
      const f32x4 w0 = *reinterpret_cast<const f32x4*>(a.w + seg.start + i);
#pragma unroll
      for (int e = 0; e < 4; ++e) w[e] = w0[e];
    } else {
      w[0] = a.w[seg.start + i];
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const double wd = static_cast<double>(w[e]);
      acc = fma(x[e], wd, acc);
      acc_abs = fma(fabs(x[e]), fabs(wd), acc_abs);
    }
  }
  acc = wave_sum(acc);
  acc_abs = wave_sum(acc_abs);
  if (lane == 0) {
    a.out[static_cast<int64_t>(si) * a.K + k] = acc;
    a.out_abs[static_cast<int64_t>(si) * a.K + k] = acc_abs;
  }
  }
}

// One workgroup per item (a run of rows of one partial block, contiguous in
// memory).  A thread walks the run in steps of the workgroup width, four
// 16-byte loads in flight; wave sums, then the four waves in order.
template <bool VEC>
__global__ __launch_bounds__(kThreads) void bilinear_kernel(BilinearArgs a) {
  __shared__ double wave_part[kThreads / 64];
  for (int64_t it = blockIdx.x; it < a.n_items; it += gridDim.x) {
    const VerifyItem item = a.items[it];
    const cleave_task task = a.tasks[item.task];
    const uint32_t n_len = task.n_len;
    const float* P = a.partials + task.partial_off + static_cast<uint64_t>(item.row0) * n_len;
    const float* rr = a.r + task.m0 + item.row0;
    const float* ss = a.s + task.n0;
    const uint32_t count = item.rows * n_len;
    double acc = 0.0;
    if constexpr (VEC) {
      constexpr uint32_t kStride = kThreads * 4;
      constexpr int U = 4;
      for (uint32_t e0 = threadIdx.x * 4; e0 < count; e0 += U * kStride) {
        f32x4 p[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const uint32_t e = e0 + u * kStride;
          p[u] = e < count ? __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(P + e))
                           : f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const uint32_t e = e0 + u * kStride;
          if (e < count) {
            const uint32_t row = e / n_len;
            const uint32_t col = e - row * n_len;
            const f32x4 s4 = *reinterpret_cast<const f32x4*>(ss + col);
            double tsum = static_cast<double>(p[u][0]) * static_cast<double>(s4[0]);
            tsum = fma(static_cast<double>(p[u][1]), static_cast<double>(s4[1]), tsum);
            tsum = fma(static_cast<double>(p[u][2]), static_cast<double>(s4[2]), tsum);
            tsum = fma(static_cast<double>(p[u][3]), static_cast<double>(s4[3]), tsum);
            acc = fma(static_cast<double>(rr[row]), tsum, acc);
          }
        }
      }
    } else {
      for (uint32_t e = threadIdx.x; e < count; e += kThreads) {
        const uint32_t row = e / n_len;
        const uint32_t col = e - row * n_len;
        acc = fma(static_cast<double>(rr[row]),
                  static_cast<double>(P[e]) * static_cast<double>(ss[col]), acc);
      }
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
      double total = 0.0;
#pragma unroll
      for (int w = 0; w < kThreads / 64; ++w) total += wave_part[w];
      a.item_sums[it] = total;
    }
    __syncthreads();   // wave_part is reused by the next item
  }
}

// One wave per task.
__global__ __launch_bounds__(kThreads) void verdict_kernel(VerdictArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t t = static_cast<int64_t>(blockIdx.x) * (kThreads / 64) + (threadIdx.x >> 6);
  if (t >= a.n_tasks) return;
  const cleave_task task = a.tasks[t];
  double lhs = 0.0;
  for (uint32_t i = a.task_first_item[t] + lane; i < a.task_first_item[t + 1]; i += 64)
    lhs += a.item_sums[i];
  const int64_t ro = static_cast<int64_t>(a.task_row_seg[t]) * a.K + task.k0;
  const int64_t co = static_cast<int64_t>(a.task_col_seg[t]) * a.K + task.k0;
  double rhs = 0.0, scale = 0.0;
  for (uint32_t k = lane; k < task.k_len; k += 64) {
    rhs = fma(a.U[ro + k], a.V[co + k], rhs);
    scale = fma(a.U_abs[ro + k], a.V_abs[co + k], scale);
  }
  lhs = wave_sum(lhs);
  rhs = wave_sum(rhs);
  scale = wave_sum(scale);
  if (lane == 0) {
    if (a.lhs) a.lhs[t] = lhs;
    if (a.rhs) a.rhs[t] = rhs;
    if (a.scale) a.scale[t] = scale;
    a.accept[t] = fabs(lhs - rhs) <= a.tol * scale ? 1 : 0;
  }
}

template <int EB, int VEC>
void launch_project_one(const ProjectArgs& a, bool reduce_contiguous, hipStream_t stream) {
  if (reduce_contiguous) {
    const dim3 grid(static_cast<unsigned>((a.K + 3) / 4), static_cast<unsigned>(a.n_segs < kMaxGridY ? a.n_segs : kMaxGridY));
    hipLaunchKernelGGL((project_rows_kernel<EB, VEC>), grid, dim3(kThreads), 0, stream, a);
  } else {
    constexpr int KW = (VEC == 1 ? 64 : 8) * VEC;
    const dim3 grid(static_cast<unsigned>((a.K + KW - 1) / KW), static_cast<unsigned>(a.n_segs < kMaxGridY ? a.n_segs : kMaxGridY));
    hipLaunchKernelGGL((project_strided_kernel<EB, VEC>), grid, dim3(kThreads), 0, stream, a);
  }
}

}  // namespace

hipError_t launch_project(const ProjectArgs& a, int dtype, bool reduce_contiguous, bool vec,
                          hipStream_t stream) {
  if (a.n_segs == 0 || a.K == 0) return hipSuccess;
  if (dtype == CLEAVE_BF16) {
    if (vec) launch_project_one<2, 8>(a, reduce_contiguous, stream);
    else launch_project_one<2, 1>(a, reduce_contiguous, stream);
  } else {
    if (vec) launch_project_one<4, 4>(a, reduce_contiguous, stream);
    else launch_project_one<4, 1>(a, reduce_contiguous, stream);
  }
  return hipGetLastError();
}

hipError_t launch_bilinear(const BilinearArgs& a, bool vec, hipStream_t stream) {
  if (a.n_items == 0) return hipSuccess;
  const dim3 grid(static_cast<unsigned>(a.n_items < (int64_t{1} << 20) ? a.n_items : (int64_t{1} << 20)));
  if (vec) hipLaunchKernelGGL((bilinear_kernel<true>), grid, dim3(kThreads), 0, stream, a);
  else hipLaunchKernelGGL((bilinear_kernel<false>), grid, dim3(kThreads), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_verdict(const VerdictArgs& a, hipStream_t stream) {
  if (a.n_tasks == 0) return hipSuccess;
  const dim3 grid(static_cast<unsigned>((a.n_tasks + 3) / 4));
  hipLaunchKernelGGL(verdict_kernel, grid, dim3(kThreads), 0, stream, a);
  return hipGetLastError();
}

}  // namespace cleave
