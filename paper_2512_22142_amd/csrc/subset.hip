// Work-item lists of subset launches, written on the device.
//
// A re-issued subset (paper Sec. 4.2, churn recovery: the unfinished shards of
// a departed device are dispatched again) is a list of task indices.  The host
// decides where each task's work items go; this kernel derives the items from
// the task records already on the device.  The (task, destination) pairs come
// in through the kernel arguments.
#include <hip/hip_runtime.h>

#include "kernels.h"
#include "plan_internal.h"

namespace cleave {

namespace {

// One wave per entry; lane l writes sub-tiles l, l + 64, ...
__global__ __launch_bounds__(64) void expand_subset_kernel(ExpandArgs args) {
  const uint32_t e = blockIdx.x;
  if (e >= args.n_entries) return;
  const SubsetEntry entry = args.entries[e];
  const cleave_task t = args.tasks[entry.task];
  const SubTiling s = sub_tiling(t, args.fine != 0);
  for (uint32_t sub = threadIdx.x; sub < s.count(); sub += 64)
    args.out[entry.dst + sub] = make_work_item(t, entry.task, s, sub);
}

}  // namespace

hipError_t launch_expand_subset(const ExpandArgs& args, hipStream_t stream) {
  if (args.n_entries == 0) return hipSuccess;
  hipLaunchKernelGGL(expand_subset_kernel, dim3(args.n_entries), dim3(64), 0, stream, args);
  return hipGetLastError();
}

}  // namespace cleave
