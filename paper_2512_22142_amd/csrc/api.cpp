// C-ABI entry points that touch the device: table upload, execute, reduce.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <new>
#include <vector>

#include "kernels.h"
#include "plan_internal.h"

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) {
  g_last_hip_error = static_cast<int>(e);
  return CLEAVE_EHIP;
}

#define CLEAVE_HIP(expr)                         \
  do {                                           \
    hipError_t e__ = (expr);                     \
    if (e__ != hipSuccess) return hip_fail(e__); \
  } while (0)

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

void free_device_tables(cleave_plan* p) {
  if (p->d_tasks) (void)hipFree(p->d_tasks);
  for (int c = 0; c < cleave::kNumTileClasses; ++c)
    if (p->d_items[c]) (void)hipFree(p->d_items[c]);
  if (p->d_reduce_items) (void)hipFree(p->d_reduce_items);
  if (p->d_subset_items) (void)hipFree(p->d_subset_items);
  p->d_tasks = nullptr;
  p->d_items[0] = p->d_items[1] = nullptr;
  p->d_reduce_items = nullptr;
  p->d_subset_items = nullptr;
  p->d_subset_capacity = 0;
  p->device = -1;
}

template <typename T>
int upload_vector(const std::vector<T>& v, T** dst) {
  *dst = nullptr;
  if (v.empty()) return CLEAVE_OK;
  hipError_t e = hipMalloc(reinterpret_cast<void**>(dst), v.size() * sizeof(T));
  if (e == hipErrorOutOfMemory) return CLEAVE_ENOMEM;
  if (e != hipSuccess) return hip_fail(e);
  CLEAVE_HIP(hipMemcpy(*dst, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice));
  return CLEAVE_OK;
}

int ensure_uploaded(cleave_plan* p) {
  int dev = 0;
  CLEAVE_HIP(hipGetDevice(&dev));
  if (p->device == dev) return CLEAVE_OK;
  if (p->device >= 0) free_device_tables(p);
  int rc = upload_vector(p->tasks, &p->d_tasks);
  for (int c = 0; rc == CLEAVE_OK && c < cleave::kNumTileClasses; ++c)
    rc = upload_vector(p->items[c], &p->d_items[c]);
  if (rc == CLEAVE_OK) rc = upload_vector(p->reduce_items, &p->d_reduce_items);
  if (rc != CLEAVE_OK) {
    free_device_tables(p);
    return rc;
  }
  p->device = dev;
  return CLEAVE_OK;
}

int compute_units(int* out) {
  static thread_local int cached_dev = -1, cached_cus = 0;
  int dev = 0;
  CLEAVE_HIP(hipGetDevice(&dev));
  if (dev != cached_dev) {
    CLEAVE_HIP(hipDeviceGetAttribute(&cached_cus, hipDeviceAttributeMultiprocessorCount, dev));
    cached_dev = dev;
  }
  *out = std::max(cached_cus, 1);
  return CLEAVE_OK;
}

const char* kernel_name(int dtype, int cls, bool vec, int transA, int transB) {
  static const char* names[2][2][5] = {
      {{"execute_f32_256x256_nn", "execute_f32_256x256_nt", "execute_f32_256x256_tn", "execute_f32_256x256_tt",
        "execute_f32_256x256_scalar"},
       {"execute_f32_128x128_nn", "execute_f32_128x128_nt", "execute_f32_128x128_tn", "execute_f32_128x128_tt",
        "execute_f32_128x128_scalar"}},
      {{"execute_bf16_256x256_nn", "execute_bf16_256x256_nt", "execute_bf16_256x256_tn", "execute_bf16_256x256_tt",
        "execute_bf16_256x256_scalar"},
       {"execute_bf16_128x128_nn", "execute_bf16_128x128_nt", "execute_bf16_128x128_tn", "execute_bf16_128x128_tt",
        "execute_bf16_128x128_scalar"}}};
  const int mode = vec ? (transA ? 2 : 0) + (transB ? 1 : 0) : 4;
  return names[dtype == CLEAVE_BF16 ? 1 : 0][cls][mode];
}

const char* direct_kernel_name(int cls, int transA, int transB) {
  static const char* names[2][4] = {
      {"execute_direct_bf16_256x256_nn", "execute_direct_bf16_256x256_nt",
       "execute_direct_bf16_256x256_tn", "execute_direct_bf16_256x256_tt"},
      {"execute_direct_bf16_128x128_nn", "execute_direct_bf16_128x128_nt",
       "execute_direct_bf16_128x128_tn", "execute_direct_bf16_128x128_tt"}};
  return names[cls][(transA ? 2 : 0) + (transB ? 1 : 0)];
}

}  // namespace

extern "C" int cleave_last_hip_error(void) { return g_last_hip_error; }

extern "C" int cleave_plan_upload(cleave_plan* plan) {
  if (!plan) return CLEAVE_EINVAL;
  return ensure_uploaded(plan);
}

extern "C" void cleave_plan_destroy(cleave_plan* plan) {
  if (!plan) return;
  if (plan->device >= 0) free_device_tables(plan);
  delete plan;
}

extern "C" int cleave_execute(cleave_plan* plan, const int64_t* task_ids, int64_t n_ids,
                              const void* A, int64_t lda, int transA, const void* B, int64_t ldb,
                              int transB, int dtype, float* partials, void* hip_stream) {
  if (!plan || !A || !B || !partials) return CLEAVE_EINVAL;
  if (dtype != CLEAVE_F32 && dtype != CLEAVE_BF16) return CLEAVE_EINVAL;
  if ((transA != 0 && transA != 1) || (transB != 0 && transB != 1)) return CLEAVE_EINVAL;
  if ((task_ids == nullptr) != (n_ids == 0) || n_ids < 0) return CLEAVE_EINVAL;
  if (lda < (transA ? plan->M : plan->K) || ldb < (transB ? plan->K : plan->N)) return CLEAVE_EINVAL;
  const int eb = dtype == CLEAVE_BF16 ? 2 : 4;
  if (!aligned(A, eb) || !aligned(B, eb) || !aligned(partials, 4)) return CLEAVE_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);

  // Work items of a subset, in the order the caller listed the tasks.
  std::vector<cleave::WorkItem> subset[cleave::kNumTileClasses];
  if (task_ids) {
    try {
      std::vector<bool> seen(plan->tasks.size(), false);
      for (int64_t i = 0; i < n_ids; ++i) {
        const int64_t id = task_ids[i];
        if (id < 0 || id >= static_cast<int64_t>(plan->tasks.size()) || seen[id]) return CLEAVE_EINVAL;
        seen[id] = true;
        cleave::append_work_items(plan->tasks[id], static_cast<uint32_t>(id), subset);
      }
    } catch (const std::bad_alloc&) {
      return CLEAVE_ENOMEM;
    }
  }

  int rc = ensure_uploaded(plan);
  if (rc != CLEAVE_OK) return rc;

  // 16-byte load path: every chunk and tile edge a multiple of 16 bytes and
  // all rows of both operands starting on 16-byte boundaries.
  const int e = 16 / eb;
  const bool vec = (e == 8 ? (plan->all_k_mult8 && plan->all_mn_mult8)
                           : (plan->all_k_mult4 && plan->all_mn_mult4)) &&
                   lda % e == 0 && ldb % e == 0 && aligned(A, 16) && aligned(B, 16) &&
                   // in-tile byte offsets are kept in 32 bits
                   lda * eb < (int64_t{1} << 22) && ldb * eb < (int64_t{1} << 22);

  const cleave::WorkItem* d_lists[cleave::kNumTileClasses] = {plan->d_items[0], plan->d_items[1]};
  int64_t counts[cleave::kNumTileClasses] = {static_cast<int64_t>(plan->items[0].size()),
                                             static_cast<int64_t>(plan->items[1].size())};
  if (task_ids) {
    // The subset tables live in a scratch buffer of the plan that a previous
    // subset launch on this stream may still be reading: wait, refill, and
    // wait for the copy so that the host vectors can go away.
    const int64_t total = static_cast<int64_t>(subset[0].size() + subset[1].size());
    CLEAVE_HIP(hipStreamSynchronize(stream));
    if (total > plan->d_subset_capacity) {
      if (plan->d_subset_items) (void)hipFree(plan->d_subset_items);
      plan->d_subset_items = nullptr;
      plan->d_subset_capacity = 0;
      hipError_t he = hipMalloc(reinterpret_cast<void**>(&plan->d_subset_items),
                                static_cast<size_t>(total) * sizeof(cleave::WorkItem));
      if (he == hipErrorOutOfMemory) return CLEAVE_ENOMEM;
      if (he != hipSuccess) return hip_fail(he);
      plan->d_subset_capacity = total;
    }
    int64_t pos = 0;
    for (int c = 0; c < cleave::kNumTileClasses; ++c) {
      counts[c] = static_cast<int64_t>(subset[c].size());
      d_lists[c] = plan->d_subset_items + pos;
      if (counts[c] > 0)
        CLEAVE_HIP(hipMemcpyAsync(plan->d_subset_items + pos, subset[c].data(),
                                  static_cast<size_t>(counts[c]) * sizeof(cleave::WorkItem),
                                  hipMemcpyHostToDevice, stream));
      pos += counts[c];
    }
    CLEAVE_HIP(hipStreamSynchronize(stream));
  }

  int64_t most = -1;
  for (int c = 0; c < cleave::kNumTileClasses; ++c) {
    if (counts[c] == 0) continue;
    cleave::ExecuteArgs args{};
    args.tasks = plan->d_tasks;
    args.items = d_lists[c];
    args.n_items = counts[c];
    args.A = A;
    args.B = B;
    args.lda = lda;
    args.ldb = ldb;
    args.transA = transA;
    args.transB = transB;
    args.partials = partials;
    const bool direct = vec && dtype == CLEAVE_BF16 &&
                        (cleave::direct_k_step() == 32 ? plan->all_klen_mult32 : plan->all_klen_mult64);
    if (direct) {
      // Persistent workgroups, as many as the chip holds at once: each walks
      // the item list with the grid as stride and fetches the head of its next
      // item while it stores the current one.
      int cus = 0;
      rc = compute_units(&cus);
      if (rc != CLEAVE_OK) return rc;
      const int64_t resident = static_cast<int64_t>(cus) * cleave::direct_workgroups_per_cu(c);
      const int grid = static_cast<int>(std::min<int64_t>(counts[c], resident));
      CLEAVE_HIP(cleave::launch_execute_direct(args, c, grid, stream));
    } else {
      // One workgroup per work item (the kernel loops only if the grid is
      // capped): the hardware dispatcher then balances uneven items and keeps
      // the workgroups that share a CU out of phase.
      constexpr int64_t kMaxGrid = int64_t{1} << 20;
      const int grid = static_cast<int>(std::min<int64_t>(counts[c], kMaxGrid));
      CLEAVE_HIP(cleave::launch_execute(args, dtype, c, vec, grid, stream));
    }
    if (counts[c] > most) {
      most = counts[c];
      plan->last_kernel = direct ? direct_kernel_name(c, transA, transB)
                                 : kernel_name(dtype, c, vec, transA, transB);
    }
  }
  return CLEAVE_OK;
}

extern "C" int cleave_reduce(cleave_plan* plan, const float* partials, void* C, int64_t ldc,
                             int out_dtype, void* hip_stream) {
  if (!plan || !partials || !C) return CLEAVE_EINVAL;
  if (out_dtype != CLEAVE_F32 && out_dtype != CLEAVE_BF16) return CLEAVE_EINVAL;
  if (ldc < plan->N) return CLEAVE_EINVAL;
  const int ob = out_dtype == CLEAVE_BF16 ? 2 : 4;
  if (!aligned(partials, 4) || !aligned(C, ob)) return CLEAVE_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);

  int rc = ensure_uploaded(plan);
  if (rc != CLEAVE_OK) return rc;
  int cus = 0;
  rc = compute_units(&cus);
  if (rc != CLEAVE_OK) return rc;

  const bool vec = plan->all_n_mult4 && ldc % 4 == 0 && aligned(partials, 16) && aligned(C, 4 * ob);
  cleave::ReduceArgs args{};
  args.tasks = plan->d_tasks;
  args.items = plan->d_reduce_items;
  args.n_items = static_cast<int64_t>(plan->reduce_items.size());
  args.partials = partials;
  args.C = C;
  args.ldc = ldc;
  const int grid = static_cast<int>(std::min<int64_t>(args.n_items, int64_t{1} << 20)); (void)cus;
  CLEAVE_HIP(cleave::launch_reduce(args, out_dtype, vec, grid, stream));
  return CLEAVE_OK;
}
