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
// The aggregation (Sec. 3.2) can ride along: the fused pass takes all splits
// of a tile together and writes their sum while it checks them, so the
// partial blocks are read once for both.
//
// Two launches:
//   pass      three independent jobs in one grid --
//             projections U[seg][k] = sum_i op(A)[i][k] r[i] over a row segment
//             (and the same with absolute values), V[seg][k] likewise for
//             op(B) and s, and per run of rows of a partial block the bilinear
//             form sum_i r_i sum_j P_ij s_j;
//   verdict   per task: lhs from its item sums, rhs = sum_k U_k V_k and
//             scale = sum_k |U|_k |V|_k over the task's chunk, and the
//             decision |lhs - rhs| <= tol * scale.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "kernels.h"

namespace cleave {

namespace {

constexpr int kThreads = 256;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

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

// VEC consecutive fp32 weights, widened.
template <int VEC>
__device__ __forceinline__ void load_weights(const float* w, double (&out)[VEC]) {
  if constexpr (VEC == 1) {
    out[0] = static_cast<double>(w[0]);
  } else {
#pragma unroll
    for (int h = 0; h < VEC / 4; ++h) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(w + 4 * h);
#pragma unroll
      for (int e = 0; e < 4; ++e) out[4 * h + e] = static_cast<double>(v[e]);
    }
  }
}

// Sum over the 64 lanes of a wave, same tree on every call.
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}

// Projection, the summed index strides through memory (x(i, k) = src[i * ld + k]).
// Unit of work: one segment x KW consecutive k.  A thread owns VEC consecutive
// k and every SL-th row of the segment; the row slices are combined first
// inside each wave (lanes that share a k chunk), then over the four waves in
// ascending order.
template <int EB, int VEC>
struct ProjectStrided {
  static constexpr int KT = VEC == 1 ? 64 : 8;   // threads along k
  static constexpr int SL = kThreads / KT;       // row slices
  static constexpr int KW = KT * VEC;            // k per unit
  static constexpr int kSmemDoubles = 2 * (kThreads / 64) * KW;

  __device__ static void run(const ProjectArgs& a, int si, int64_t kblock, double* smem) {
    const int member = si / a.n_segs;
    const Segment seg = a.segs[si - member * a.n_segs];
    const int64_t moff = member_offset(a.at, a.batch, static_cast<uint32_t>(member));
    const float* wv = a.w + member * a.w_stride;
    const int t = threadIdx.x;
    const int kc = t % KT;
    const int slice = t / KT;
    const int64_t k = kblock * KW + kc * VEC;
    double acc[VEC], acc_abs[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = acc_abs[e] = 0.0;
    if (k < a.K) {
#pragma unroll 4
      for (uint32_t i = slice; i < seg.len; i += SL) {
        const int64_t row = static_cast<int64_t>(seg.start) + i;
        const double w = static_cast<double>(wv[row]);
        double x[VEC];
        load_elems<EB, VEC>(a.src, moff + row * a.ld + k, x);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          acc[e] = fma(x[e], w, acc[e]);
          acc_abs[e] = fma(fabs(x[e]), fabs(w), acc_abs[e]);
        }
      }
    }
    // lanes l, l + KT, l + 2 KT, ... of a wave hold the same k chunk
#pragma unroll
    for (int m = 32; m >= KT; m >>= 1) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        acc[e] += __shfl_xor(acc[e], m, 64);
        acc_abs[e] += __shfl_xor(acc_abs[e], m, 64);
      }
    }
    const int wave = t >> 6, lane = t & 63;
    if (KT == 64 || lane < KT) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        smem[(0 * (kThreads / 64) + wave) * KW + (lane % KT) * VEC + e] = acc[e];
        smem[(1 * (kThreads / 64) + wave) * KW + (lane % KT) * VEC + e] = acc_abs[e];
      }
    }
    __syncthreads();
    if (t < KW) {
      const int64_t ko = kblock * KW + t;
      if (ko < a.K) {
        double s0 = 0.0, s1 = 0.0;
#pragma unroll
        for (int w = 0; w < kThreads / 64; ++w) {
          s0 += smem[(0 * (kThreads / 64) + w) * KW + t];
          s1 += smem[(1 * (kThreads / 64) + w) * KW + t];
        }
        a.out[static_cast<int64_t>(si) * a.K + ko] = s0;
        a.out_abs[static_cast<int64_t>(si) * a.K + ko] = s1;
      }
    }
    __syncthreads();   // smem is reused by the workgroup's next unit
  }
};

// Projection, the summed index is contiguous (x(i, k) = src[k * ld + i]).
// Unit of work: one segment x KW consecutive k.  A wave reads 8 k rows at a
// time, 8 lanes per row (8 x VEC contiguous elements per load and row); the 8
// lanes of a row are combined by a fixed 3-step tree.
template <int EB, int VEC>
struct ProjectRows {
  static constexpr int LPR = 8;                  // lanes per k row
  static constexpr int RPW = 64 / LPR;           // k rows per wave and round
  static constexpr int ROUNDS = 2;
  static constexpr int KW = (kThreads / 64) * RPW * ROUNDS;
  static constexpr int kSmemDoubles = 0;

  __device__ static void run(const ProjectArgs& a, int si, int64_t kblock, double*) {
    const int member = si / a.n_segs;
    const Segment seg = a.segs[si - member * a.n_segs];
    const int64_t moff = member_offset(a.at, a.batch, static_cast<uint32_t>(member));
    const float* wv = a.w + member * a.w_stride;
    const int lane = threadIdx.x & 63;
    const int c = lane % LPR;
    for (int round = 0; round < ROUNDS; ++round) {
      const int64_t k = kblock * KW + ((threadIdx.x >> 6) * ROUNDS + round) * RPW + lane / LPR;
      // rows past K are read as row K-1 (no out-of-range access) and not stored
      const int64_t base = moff + (k < a.K ? k : a.K - 1) * a.ld + seg.start;
      double acc = 0.0, acc_abs = 0.0;
#pragma unroll 4
      for (uint32_t i = c * VEC; i < seg.len; i += LPR * VEC) {
        double x[VEC], w[VEC];
        load_elems<EB, VEC>(a.src, base + i, x);
        load_weights<VEC>(wv + seg.start + i, w);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          acc = fma(x[e], w[e], acc);
          acc_abs = fma(fabs(x[e]), fabs(w[e]), acc_abs);
        }
      }
#pragma unroll
      for (int m = LPR / 2; m >= 1; m >>= 1) {
        acc += __shfl_xor(acc, m, 64);
        acc_abs += __shfl_xor(acc_abs, m, 64);
      }
      if (c == 0 && k < a.K) {
        a.out[static_cast<int64_t>(si) * a.K + k] = acc;
        a.out_abs[static_cast<int64_t>(si) * a.K + k] = acc_abs;
      }
    }
  }
};

// Bilinear form over one item (a run of rows of one partial block, contiguous
// in memory).  A thread walks the run in steps of the workgroup width, eight
// 16-byte loads in flight; wave sums, then the four waves in order.
template <bool VEC>
__device__ __forceinline__ void bilinear_item(const BilinearArgs& a, int64_t it, double* smem) {
  const VerifyItem item = a.items[it];
  const cleave_task task = a.tasks[item.task];
  const uint32_t n_len = task.n_len;
  const float* P = a.partials + task.partial_off + static_cast<uint64_t>(item.row0) * n_len;
  const int64_t member = a.batched ? task.gemm_id : 0;
  const float* rr = a.r + member * a.r_stride + task.m0 + item.row0;
  const float* ss = a.s + member * a.s_stride + task.n0;
  const uint32_t count = item.rows * n_len;
  double acc = 0.0;
  if constexpr (VEC) {
    constexpr uint32_t kStride = kThreads * 4;
    constexpr int U = 8;
    // (row, column) of a thread's element advance by a fixed step per load:
    // one division per item instead of one per load.
    const uint32_t q = kStride / n_len, rem = kStride - q * n_len;
    uint32_t e = threadIdx.x * 4;
    uint32_t row = e / n_len;
    uint32_t col = e - row * n_len;
    while (e < count) {
      f32x4 p[U];
      uint32_t rows[U], cols[U];
      bool valid[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        valid[u] = e < count;
        p[u] = valid[u] ? __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(P + e))
                        : f32x4{0.f, 0.f, 0.f, 0.f};
        rows[u] = row;
        cols[u] = col;
        e += kStride;
        row += q;
        col += rem;
        if (col >= n_len) {
          col -= n_len;
          ++row;
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (valid[u]) {
          const f32x4 s4 = *reinterpret_cast<const f32x4*>(ss + cols[u]);
          double tsum = static_cast<double>(p[u][0]) * static_cast<double>(s4[0]);
          tsum = fma(static_cast<double>(p[u][1]), static_cast<double>(s4[1]), tsum);
          tsum = fma(static_cast<double>(p[u][2]), static_cast<double>(s4[2]), tsum);
          tsum = fma(static_cast<double>(p[u][3]), static_cast<double>(s4[3]), tsum);
          acc = fma(static_cast<double>(rr[rows[u]]), tsum, acc);
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
  if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double total = 0.0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) total += smem[w];
    a.item_sums[it] = total;
  }
  __syncthreads();   // smem is reused by the workgroup's next unit
}

template <bool C, typename T, typename F>
struct pick { typedef T type; };
template <typename T, typename F>
struct pick<false, T, F> { typedef F type; };

// One launch for the three independent jobs: projection units of A, of B, and
// the bilinear items share one list of units that the workgroups walk with the
// grid as stride.
template <int EB, bool VEC, bool A_CONTIG, bool B_CONTIG>
__global__ __launch_bounds__(kThreads) void verify_pass_kernel(VerifyPassArgs a) {
  constexpr int V = VEC ? 16 / EB : 1;
  typedef typename pick<A_CONTIG, ProjectRows<EB, V>, ProjectStrided<EB, V>>::type ProjA;
  typedef typename pick<B_CONTIG, ProjectRows<EB, V>, ProjectStrided<EB, V>>::type ProjB;
  constexpr int kSmem = ProjA::kSmemDoubles > ProjB::kSmemDoubles ? ProjA::kSmemDoubles
                                                                   : ProjB::kSmemDoubles;
  __shared__ double smem[kSmem > 8 ? kSmem : 8];
  const int64_t kbA = (a.A.K + ProjA::KW - 1) / ProjA::KW;
  const int64_t kbB = (a.B.K + ProjB::KW - 1) / ProjB::KW;
  const int64_t unitsA = kbA * a.A.n_segs * a.A.n_members;
  const int64_t unitsB = kbB * a.B.n_segs * a.B.n_members;
  const int64_t proj = unitsA + unitsB;
  const int64_t total = proj + a.bil.n_items;
  // every `every`-th unit is a projection unit until they are used up, so that
  // the compute-heavier projections are spread over the item stream
  const int64_t every = proj > 0 ? total / proj : 1;
  for (int64_t u = blockIdx.x; u < total; u += gridDim.x) {
    const int64_t slot = u / every;
    if (u % every == 0 && slot < proj) {
      if (slot < unitsA) {
        ProjA::run(a.A, static_cast<int>(slot / kbA), slot % kbA, smem);
      } else {
        const int64_t v = slot - unitsA;
        ProjB::run(a.B, static_cast<int>(v / kbB), v % kbB, smem);
      }
    } else {
      const int64_t before = (u + every - 1) / every;   // projection slots below u
      bilinear_item<VEC>(a.bil, u - (before < proj ? before : proj), smem);
    }
  }
}

// Round-to-nearest-even fp32 -> bf16 (NaN stays a quiet NaN).
__device__ __forceinline__ uint32_t to_bf16_bits(float x) {
  uint32_t u = __builtin_bit_cast(uint32_t, x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

// The bilinear items of all S splits of a tile over one run of rows, and the
// tile's aggregated rows into C (paper Sec. 3.2 and Sec. 6: the PS checks the
// returned blocks and aggregates them).  Per split the arithmetic and the
// combination over lanes and waves are those of bilinear_item (over a shorter
// run of rows); the fold over the splits is the aggregation kernel's,
// ((P0 + P1) + P2) + ..., plain fp32 adds.
template <bool VEC, int S>
__device__ __forceinline__ void aggregate_item(const BilinearArgs& a, const AggregateArgs& g,
                                               const VerifyItem& item, double* smem) {
  const cleave_task task = a.tasks[item.task];            // the tile's first split
  const uint32_t n_len = task.n_len;
  const uint64_t block = static_cast<uint64_t>(task.m_len) * n_len;   // elements between two splits' blocks
  const float* P = a.partials + task.partial_off + static_cast<uint64_t>(item.row0) * n_len;
  const float* rr = a.r + task.m0 + item.row0;
  const float* ss = a.s + task.n0;
  const int64_t c_at = static_cast<int64_t>(task.m0 + item.row0) * g.ldc + task.n0;
  const uint32_t count = item.rows * n_len;
  double acc[S];
#pragma unroll
  for (int sp = 0; sp < S; ++sp) acc[sp] = 0.0;
  if constexpr (VEC) {
    constexpr uint32_t kStride = kThreads * 4;
    constexpr int U = S <= 2 ? 8 : (S <= 4 ? 4 : 2);      // 16 loads of 16 bytes in flight per thread
    const uint32_t q = kStride / n_len, rem = kStride - q * n_len;
    uint32_t e = threadIdx.x * 4;
    uint32_t row = e / n_len;
    uint32_t col = e - row * n_len;
    while (e < count) {
      f32x4 p[U][S];
      uint32_t rows[U], cols[U];
      bool valid[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        valid[u] = e < count;
#pragma unroll
        for (int sp = 0; sp < S; ++sp)
          p[u][sp] = valid[u] ? __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(P + sp * block + e))
                              : f32x4{0.f, 0.f, 0.f, 0.f};
        rows[u] = row;
        cols[u] = col;
        e += kStride;
        row += q;
        col += rem;
        if (col >= n_len) {
          col -= n_len;
          ++row;
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (valid[u]) {
          const f32x4 s4 = *reinterpret_cast<const f32x4*>(ss + cols[u]);
          const double rv = static_cast<double>(rr[rows[u]]);
#pragma unroll
          for (int sp = 0; sp < S; ++sp) {
            double tsum = static_cast<double>(p[u][sp][0]) * static_cast<double>(s4[0]);
            tsum = fma(static_cast<double>(p[u][sp][1]), static_cast<double>(s4[1]), tsum);
            tsum = fma(static_cast<double>(p[u][sp][2]), static_cast<double>(s4[2]), tsum);
            tsum = fma(static_cast<double>(p[u][sp][3]), static_cast<double>(s4[3]), tsum);
            acc[sp] = fma(rv, tsum, acc[sp]);
          }
          f32x4 sum = p[u][0];
#pragma unroll
          for (int sp = 1; sp < S; ++sp) sum = sum + p[u][sp];
          const int64_t off = c_at + static_cast<int64_t>(rows[u]) * g.ldc + cols[u];
          if (g.out_bf16) {
            u32x2 w;
            w[0] = to_bf16_bits(sum[0]) | (to_bf16_bits(sum[1]) << 16);
            w[1] = to_bf16_bits(sum[2]) | (to_bf16_bits(sum[3]) << 16);
            *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(g.C) + off) = w;
          } else {
            *reinterpret_cast<f32x4*>(static_cast<float*>(g.C) + off) = sum;
          }
        }
      }
    }
  } else {
    for (uint32_t e = threadIdx.x; e < count; e += kThreads) {
      const uint32_t row = e / n_len;
      const uint32_t col = e - row * n_len;
      const double rv = static_cast<double>(rr[row]);
      const double sv = static_cast<double>(ss[col]);
      float sum = 0.0f;
#pragma unroll
      for (int sp = 0; sp < S; ++sp) {
        const float pv = P[sp * block + e];
        acc[sp] = fma(rv, static_cast<double>(pv) * sv, acc[sp]);
        sum = sp == 0 ? pv : sum + pv;
      }
      const int64_t off = c_at + static_cast<int64_t>(row) * g.ldc + col;
      if (g.out_bf16) static_cast<uint16_t*>(g.C)[off] = static_cast<uint16_t>(to_bf16_bits(sum));
      else static_cast<float*>(g.C)[off] = sum;
    }
  }
#pragma unroll
  for (int sp = 0; sp < S; ++sp) {
    const double w = wave_sum(acc[sp]);
    if ((threadIdx.x & 63) == 0) smem[sp * (kThreads / 64) + (threadIdx.x >> 6)] = w;
  }
  __syncthreads();
  if (threadIdx.x < S) {
    const uint32_t ipt = g.first_item[item.task + 1] - g.first_item[item.task];   // slots per task
    double total = 0.0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) total += smem[threadIdx.x * (kThreads / 64) + w];
    a.item_sums[item.slot + threadIdx.x * ipt] = total;
  }
  __syncthreads();   // smem is reused by the workgroup's next unit
}

template <bool VEC>
__device__ __forceinline__ void aggregate_item_any(const BilinearArgs& a, const AggregateArgs& g, int64_t idx,
                                                   double* smem) {
  const VerifyItem it0 = g.items[idx];
  switch (a.tasks[it0.task].ksplit_cnt) {               // uniform over the workgroup
    case 1: aggregate_item<VEC, 1>(a, g, it0, smem); break;
    case 2: aggregate_item<VEC, 2>(a, g, it0, smem); break;
    case 3: aggregate_item<VEC, 3>(a, g, it0, smem); break;
    case 4: aggregate_item<VEC, 4>(a, g, it0, smem); break;
    case 5: aggregate_item<VEC, 5>(a, g, it0, smem); break;
    case 6: aggregate_item<VEC, 6>(a, g, it0, smem); break;
    case 7: aggregate_item<VEC, 7>(a, g, it0, smem); break;
    default: aggregate_item<VEC, 8>(a, g, it0, smem); break;   // the caller admits at most kMaxFusedSplits
  }
}

// The pass with the aggregation folded in: projection units and tile items in
// one grid, spread as in verify_pass_kernel.
template <int EB, bool VEC, bool A_CONTIG, bool B_CONTIG>
__global__ __launch_bounds__(kThreads) void verify_reduce_pass_kernel(VerifyReducePassArgs a) {
  constexpr int V = VEC ? 16 / EB : 1;
  typedef typename pick<A_CONTIG, ProjectRows<EB, V>, ProjectStrided<EB, V>>::type ProjA;
  typedef typename pick<B_CONTIG, ProjectRows<EB, V>, ProjectStrided<EB, V>>::type ProjB;
  constexpr int kProjSmem = ProjA::kSmemDoubles > ProjB::kSmemDoubles ? ProjA::kSmemDoubles
                                                                       : ProjB::kSmemDoubles;
  constexpr int kAggSmem = kMaxFusedSplits * (kThreads / 64);
  __shared__ double smem[kProjSmem > kAggSmem ? kProjSmem : kAggSmem];
  const int64_t kbA = (a.A.K + ProjA::KW - 1) / ProjA::KW;
  const int64_t kbB = (a.B.K + ProjB::KW - 1) / ProjB::KW;
  const int64_t unitsA = kbA * a.A.n_segs * a.A.n_members;
  const int64_t unitsB = kbB * a.B.n_segs * a.B.n_members;
  const int64_t proj = unitsA + unitsB;
  const int64_t total = proj + a.agg.n_items;
  const int64_t every = proj > 0 ? total / proj : 1;
  for (int64_t u = blockIdx.x; u < total; u += gridDim.x) {
    const int64_t slot = u / every;
    if (u % every == 0 && slot < proj) {
      if (slot < unitsA) {
        ProjA::run(a.A, static_cast<int>(slot / kbA), slot % kbA, smem);
      } else {
        const int64_t v = slot - unitsA;
        ProjB::run(a.B, static_cast<int>(v / kbB), v % kbB, smem);
      }
    } else {
      const int64_t before = (u + every - 1) / every;   // projection slots below u
      aggregate_item_any<VEC>(a.bil, a.agg, u - (before < proj ? before : proj), smem);
    }
  }
}

// One workgroup per task; wave sums, then the four waves in order.
__global__ __launch_bounds__(kThreads) void verdict_kernel(VerdictArgs a) {
  __shared__ double part[3][kThreads / 64];
  for (int64_t t = blockIdx.x; t < a.n_tasks; t += gridDim.x) {
  const cleave_task task = a.tasks[t];
  double lhs = 0.0;
  for (uint32_t i = a.task_first_item[t] + threadIdx.x; i < a.task_first_item[t + 1]; i += kThreads)
    lhs += a.item_sums[i];
  const int64_t member = a.batched ? task.gemm_id : 0;
  const int64_t ro = (member * a.n_row_segs + a.task_row_seg[t]) * a.K + task.k0;
  const int64_t co = (member * a.n_col_segs + a.task_col_seg[t]) * a.K + task.k0;
  double rhs = 0.0, scale = 0.0;
  for (uint32_t k = threadIdx.x; k < task.k_len; k += kThreads) {
    rhs = fma(a.U[ro + k], a.V[co + k], rhs);
    scale = fma(a.U_abs[ro + k], a.V_abs[co + k], scale);
  }
  lhs = wave_sum(lhs);
  rhs = wave_sum(rhs);
  scale = wave_sum(scale);
  if ((threadIdx.x & 63) == 0) {
    part[0][threadIdx.x >> 6] = lhs;
    part[1][threadIdx.x >> 6] = rhs;
    part[2][threadIdx.x >> 6] = scale;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    lhs = rhs = scale = 0.0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
      lhs += part[0][w];
      rhs += part[1][w];
      scale += part[2][w];
    }
    if (a.lhs) a.lhs[t] = lhs;
    if (a.rhs) a.rhs[t] = rhs;
    if (a.scale) a.scale[t] = scale;
    a.accept[t] = fabs(lhs - rhs) <= a.tol * scale ? 1 : 0;
  }
  __syncthreads();   // part is reused by the next task
  }
}

template <int EB, bool VEC>
void launch_pass_layouts(const VerifyPassArgs& a, bool a_contig, bool b_contig, dim3 grid,
                         hipStream_t stream) {
  const dim3 block(kThreads);
  if (a_contig && b_contig)
    hipLaunchKernelGGL((verify_pass_kernel<EB, VEC, true, true>), grid, block, 0, stream, a);
  else if (a_contig)
    hipLaunchKernelGGL((verify_pass_kernel<EB, VEC, true, false>), grid, block, 0, stream, a);
  else if (b_contig)
    hipLaunchKernelGGL((verify_pass_kernel<EB, VEC, false, true>), grid, block, 0, stream, a);
  else
    hipLaunchKernelGGL((verify_pass_kernel<EB, VEC, false, false>), grid, block, 0, stream, a);
}

}  // namespace

hipError_t launch_verify_pass(const VerifyPassArgs& a, int dtype, bool a_contig, bool b_contig,
                              bool vec, hipStream_t stream) {
  // k per projection unit: the same for every element type and vector width
  constexpr int kwRows = ProjectRows<2, 8>::KW, kwStrided = ProjectStrided<2, 8>::KW;
  static_assert(ProjectRows<4, 1>::KW == kwRows && ProjectStrided<4, 1>::KW == kwStrided &&
                ProjectStrided<4, 4>::KW <= kwStrided, "grid size below assumes these");
  const int64_t kbA = (a.A.K + (a_contig ? kwRows : kwStrided / 2) - 1) / (a_contig ? kwRows : kwStrided / 2);
  const int64_t kbB = (a.B.K + (b_contig ? kwRows : kwStrided / 2) - 1) / (b_contig ? kwRows : kwStrided / 2);
  // (an upper bound for the strided fp32 vector case, exact otherwise up to a factor 2)
  const int64_t units = kbA * a.A.n_segs * a.A.n_members + kbB * a.B.n_segs * a.B.n_members + a.bil.n_items;
  if (units == 0) return hipSuccess;
  const dim3 grid(static_cast<unsigned>(units < (int64_t{1} << 20) ? units : (int64_t{1} << 20)));
  if (dtype == CLEAVE_BF16) {
    if (vec) launch_pass_layouts<2, true>(a, a_contig, b_contig, grid, stream);
    else launch_pass_layouts<2, false>(a, a_contig, b_contig, grid, stream);
  } else {
    if (vec) launch_pass_layouts<4, true>(a, a_contig, b_contig, grid, stream);
    else launch_pass_layouts<4, false>(a, a_contig, b_contig, grid, stream);
  }
  return hipGetLastError();
}

namespace {

template <int EB, bool VEC>
void launch_fused_layouts(const VerifyReducePassArgs& a, bool a_contig, bool b_contig, dim3 grid,
                          hipStream_t stream) {
  const dim3 block(kThreads);
  if (a_contig && b_contig)
    hipLaunchKernelGGL((verify_reduce_pass_kernel<EB, VEC, true, true>), grid, block, 0, stream, a);
  else if (a_contig)
    hipLaunchKernelGGL((verify_reduce_pass_kernel<EB, VEC, true, false>), grid, block, 0, stream, a);
  else if (b_contig)
    hipLaunchKernelGGL((verify_reduce_pass_kernel<EB, VEC, false, true>), grid, block, 0, stream, a);
  else
    hipLaunchKernelGGL((verify_reduce_pass_kernel<EB, VEC, false, false>), grid, block, 0, stream, a);
}

}  // namespace

hipError_t launch_verify_reduce_pass(const VerifyReducePassArgs& a, int dtype, bool a_contig, bool b_contig,
                                     bool vec, hipStream_t stream) {
  constexpr int kwRows = ProjectRows<2, 8>::KW, kwStrided = ProjectStrided<2, 8>::KW;
  const int64_t kbA = (a.A.K + (a_contig ? kwRows : kwStrided / 2) - 1) / (a_contig ? kwRows : kwStrided / 2);
  const int64_t kbB = (a.B.K + (b_contig ? kwRows : kwStrided / 2) - 1) / (b_contig ? kwRows : kwStrided / 2);
  const int64_t units = kbA * a.A.n_segs * a.A.n_members + kbB * a.B.n_segs * a.B.n_members + a.agg.n_items;
  if (units == 0) return hipSuccess;
  const dim3 grid(static_cast<unsigned>(units < (int64_t{1} << 20) ? units : (int64_t{1} << 20)));
  if (dtype == CLEAVE_BF16) {
    if (vec) launch_fused_layouts<2, true>(a, a_contig, b_contig, grid, stream);
    else launch_fused_layouts<2, false>(a, a_contig, b_contig, grid, stream);
  } else {
    if (vec) launch_fused_layouts<4, true>(a, a_contig, b_contig, grid, stream);
    else launch_fused_layouts<4, false>(a, a_contig, b_contig, grid, stream);
  }
  return hipGetLastError();
}

hipError_t launch_verdict(const VerdictArgs& a, hipStream_t stream) {
  if (a.n_tasks == 0) return hipSuccess;
  const dim3 grid(static_cast<unsigned>(a.n_tasks < (int64_t{1} << 20) ? a.n_tasks : (int64_t{1} << 20)));
  hipLaunchKernelGGL(verdict_kernel, grid, dim3(kThreads), 0, stream, a);
  return hipGetLastError();
}

}  // namespace cleave
