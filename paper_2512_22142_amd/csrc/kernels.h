// Launch interface between the C-ABI layer and the HIP kernels.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "plan_internal.h"

namespace cleave {

// Most members a grouped launch (one table entry per member) can have.
constexpr int kMaxGroup = 8;

// Where batch member g's matrix starts, as an element offset from the base
// pointer.  Strided batch (batch_inner > 0): member o * batch_inner + i at
// o * outer + i * inner.  Grouped launch (n_group > 0): member g at table[g].
// Plain plans have one member at offset 0.
struct MemberOffsets {
  int64_t outer, inner;
  int64_t table[kMaxGroup];
};

struct BatchShape {
  uint32_t batch_inner;
  uint32_t n_group;
};

__host__ __device__ inline int64_t member_offset(const MemberOffsets& at, BatchShape b, uint32_t gemm_id) {
  if (b.n_group != 0) return at.table[gemm_id];
  if (b.batch_inner == 0) return 0;
  const uint32_t o = gemm_id / b.batch_inner;
  return static_cast<int64_t>(o) * at.outer + static_cast<int64_t>(gemm_id - o * b.batch_inner) * at.inner;
}

struct ExecuteArgs {
  const WorkItem* items;      // device work items of one tile class (self-contained records)
  int64_t n_items;
  const void* A;
  const void* B;
  int64_t lda, ldb;           // elements
  int transA, transB;
  float* partials;
  // Batched plans: task.gemm_id selects the member's operands (and, in
  // assemble mode, its output) through these offsets.
  BatchShape batch;
  MemberOffsets a_at, b_at, c_at;
  // Assemble mode (C != nullptr): blocks go straight to their place in the
  // output matrix (fp32, or bf16 when c_bf16 != 0) instead of `partials`.
  void* C;
  int64_t ldc;
  int c_bf16;
  // The output (partials, or C in assemble mode) takes a 16-byte (fp32) or
  // 8-byte (bf16) store at every fourth column of every sub-tile row.
  int out_vec;
  // Direct kernel only.  Null: workgroup b takes items b, b + grid, ...
  // Otherwise grid + 1 entries: workgroup b takes items [wg_ranges[b], wg_ranges[b + 1]).
  const uint32_t* wg_ranges;
};

// Enqueues the execute kernel for one tile class.  `vec` selects the 16-byte
// load path (caller has checked alignment and divisibility).
hipError_t launch_execute(const ExecuteArgs& args, int dtype, int tile_class, bool vec, int grid,
                          hipStream_t stream);

// Enqueues the bf16 direct-to-LDS execute kernel for one tile class.  The
// caller has checked the 16-byte load conditions and that the chunk length of
// every item is a multiple of kDirectKStep elements.
hipError_t launch_execute_direct(const ExecuteArgs& args, int tile_class, int grid,
                                 hipStream_t stream);
// Workgroups of the direct kernel that one CU holds at a time, per tile class.
int direct_workgroups_per_cu(int tile_class);

// Raises the dynamic-LDS limit of every execute kernel on the current device
// (needed once per device and process, before the first launch).
hipError_t configure_execute_kernels();
hipError_t configure_execute_direct_kernels();

// ---- work-item lists of subset launches ---------------------------------------
// One entry per re-issued task: which task, and where its work items go.  The
// entries travel in the kernel arguments, so the launch needs no host buffer,
// no copy and nothing the caller could not capture into a HIP graph.
struct SubsetEntry {
  uint32_t task;   // index into the task table
  uint32_t dst;    // index of the task's first work item in `out`
};
constexpr int kSubsetEntriesPerLaunch = 480;
struct ExpandArgs {
  const cleave_task* tasks;
  WorkItem* out;
  uint32_t n_entries;
  uint32_t fine;             // every block cut into small-class sub-tiles
  SubsetEntry entries[kSubsetEntriesPerLaunch];
};
static_assert(sizeof(ExpandArgs) <= 4096, "kernel arguments stay within 4 KB");
// out[dst + sub] = work item `sub` of entries[e].task, for every entry.
hipError_t launch_expand_subset(const ExpandArgs& args, hipStream_t stream);

struct ReduceArgs {
  const cleave_task* tasks;
  const ReduceItem* items;
  int64_t n_items;
  const float* partials;
  void* C;
  int64_t ldc;                // elements
  BatchShape batch;           // as in ExecuteArgs; offsets apply to C
  MemberOffsets c_at;
};

// Enqueues the aggregation kernel.  `vec` selects the float4 path.
hipError_t launch_reduce(const ReduceArgs& args, int out_dtype, bool vec, int grid,
                         hipStream_t stream);

// Aggregation with a residual added: C = sum of partials + R; R has C's
// element type, leading dimension and batch strides.
hipError_t launch_reduce_residual(const ReduceArgs& args, const void* R, int out_dtype, bool vec,
                                  int grid, hipStream_t stream);

// Aggregation feeding an Adam update of the weight whose gradient the sum is
// (ReduceArgs::C unused; w, m, v, w_bf16 share ldc and the batch strides).
struct AdamArgs {
  float* w;
  float* m;
  float* v;
  uint16_t* w_bf16;   // may be null
  float lr, beta1, beta2, eps, weight_decay;
  float inv_bias1, inv_bias2;   // 1 / (1 - beta^step)
};
hipError_t launch_reduce_adam(const ReduceArgs& args, const AdamArgs& h, bool vec, int grid,
                              hipStream_t stream);
// Grouped form: h holds member 0's arrays, `at` the element offsets of member
// g's arrays from them (ReduceArgs::c_at must be all zero: every array has its
// own table).
struct AdamGroupOffsets {
  int64_t w[kMaxGroup], m[kMaxGroup], v[kMaxGroup], w_bf16[kMaxGroup];
};
hipError_t launch_reduce_adam_grouped(const ReduceArgs& args, const AdamArgs& h, const AdamGroupOffsets& at,
                                      bool vec, int grid, hipStream_t stream);

// ---- returned-block check ---------------------------------------------------

// Projection of a stored operand onto a weight vector, once per segment:
//   out[seg][k]     = sum_{i in seg} x(i, k) * w[seg.start + i]
//   out_abs[seg][k] = sum_{i in seg} |x(i, k)| * |w[seg.start + i]|
// for k in [0, K).  reduce_contiguous = false: x(i, k) = src[i * ld + k] (the
// summed index strides, k is contiguous); true: x(i, k) = src[k * ld + i].
// Batched plans: the projection is made once per (member, segment); member g's
// operand starts member_offset(at, batch, g) elements after src, its weights
// g * w_stride entries after w, and its outputs follow member g-1's (index
// (g * n_segs + seg) * K + k).  Plain plans: n_members = 1, offsets zero.
struct ProjectArgs {
  const void* src;
  int64_t ld;               // elements
  const Segment* segs;
  int n_segs;
  const float* w;
  double* out;
  double* out_abs;
  int64_t K;
  int n_members;
  int64_t w_stride;
  BatchShape batch;
  MemberOffsets at;
};

// item_sums[item] = sum_{rows of the item} r[m0 + i] * sum_j P[i][j] * s[n0 + j].
// Batched plans (batched != 0): task.gemm_id selects the member's probe vectors,
// r_stride / s_stride entries apart.
struct BilinearArgs {
  const cleave_task* tasks;
  const VerifyItem* items;
  int64_t n_items;
  const float* partials;
  const float* r;
  const float* s;
  double* item_sums;
  int batched;
  int64_t r_stride, s_stride;
};

// The two projections and the bilinear items in one launch.  a_contig /
// b_contig: the summed index of that operand is the contiguous one.  `vec`
// selects 16-byte loads for all three jobs (caller has checked alignment and
// divisibility for all of them).
struct VerifyPassArgs {
  ProjectArgs A, B;
  BilinearArgs bil;
};
hipError_t launch_verify_pass(const VerifyPassArgs& args, int dtype, bool a_contig, bool b_contig,
                              bool vec, hipStream_t stream);

// The same pass with the aggregation folded in: a run of rows of a tile is
// taken for all of the tile's splits at once (the S blocks of a tile are
// adjacent, each m_len * n_len elements), so that every partial element is
// read once for both its check and the sum.  The runs are shorter than the
// bilinear items of the separate pass (the pass also writes; short items
// measured 15-25 % faster).  An item names the tile's first task; its sum for
// split s goes to item_sums[item.slot + s * ipt], ipt = the task's slot count
// (first_item[task + 1] - first_item[task]); C gets the left fold
// ((P0 + P1) + ...) + P_{S-1} in fp32.  Splits per tile: at most kMaxFusedSplits.
constexpr int kMaxFusedSplits = 8;
struct AggregateArgs {
  const VerifyItem* items;
  int64_t n_items;
  const uint32_t* first_item;     // per task: first slot; n_tasks + 1 entries
  void* C;
  int64_t ldc;                    // elements
  int out_bf16;
};
struct VerifyReducePassArgs {
  ProjectArgs A, B;
  BilinearArgs bil;
  AggregateArgs agg;
};
hipError_t launch_verify_reduce_pass(const VerifyReducePassArgs& args, int dtype, bool a_contig,
                                     bool b_contig, bool vec, hipStream_t stream);

// Per task: lhs = sum of its item sums (ascending), rhs = sum_k U[k] V[k] and
// scale = sum_k |U|[k] |V|[k] over the task's chunk, accept = |lhs - rhs| <= tol * scale.
struct VerdictArgs {
  const cleave_task* tasks;
  int64_t n_tasks;
  const uint32_t* task_row_seg;
  const uint32_t* task_col_seg;
  const uint32_t* task_first_item;
  const double* item_sums;
  const double* U;
  const double* U_abs;
  const double* V;
  const double* V_abs;
  int64_t K;
  int batched;          // task.gemm_id selects the member's projections
  int n_row_segs, n_col_segs;
  double tol;
  double* lhs;      // any of lhs, rhs, scale may be null
  double* rhs;
  double* scale;
  int32_t* accept;
};
hipError_t launch_verdict(const VerdictArgs& args, hipStream_t stream);

}  // namespace cleave
