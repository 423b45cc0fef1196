// Launch interface between the C-ABI layer and the HIP kernels.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "plan_internal.h"

namespace cleave {

struct ExecuteArgs {
  const cleave_task* tasks;   // device task table
  const WorkItem* items;      // device work items of one tile class
  int64_t n_items;
  const void* A;
  const void* B;
  int64_t lda, ldb;           // elements
  int transA, transB;
  float* partials;
};

// Enqueues the execute kernel for one tile class.  `vec` selects the 16-byte
// load path (caller has checked alignment and divisibility).
hipError_t launch_execute(const ExecuteArgs& args, int dtype, int tile_class, bool vec, int grid,
                          hipStream_t stream);

// Enqueues the bf16 direct-to-LDS execute kernel for one tile class.  The
// caller has checked the 16-byte load conditions and that every chunk length
// is a multiple of direct_k_step() elements.
hipError_t launch_execute_direct(const ExecuteArgs& args, int tile_class, int grid,
                                 hipStream_t stream);
// Workgroups of the direct kernel that one CU holds at a time, per tile class.
int direct_workgroups_per_cu(int tile_class);
// Elements of K the direct kernel consumes per step: chunk lengths must be multiples of it.
int direct_k_step();

struct ReduceArgs {
  const cleave_task* tasks;
  const ReduceItem* items;
  int64_t n_items;
  const float* partials;
  void* C;
  int64_t ldc;                // elements
};

// Enqueues the aggregation kernel.  `vec` selects the float4 path.
hipError_t launch_reduce(const ReduceArgs& args, int out_dtype, bool vec, int grid,
                         hipStream_t stream);

}  // namespace cleave
