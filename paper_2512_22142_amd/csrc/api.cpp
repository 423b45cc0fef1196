// C-ABI entry points that touch the device: table upload, execute, reduce.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <map>
#include <mutex>
#include <new>
#include <utility>
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

void free_verify_device(cleave::VerifyTables* v) {
  if (!v) return;
  void* ptrs[] = {v->d_row_segs, v->d_col_segs, v->d_task_row_seg, v->d_task_col_seg,
                  v->d_items, v->d_task_first_item, v->d_agg_items, v->d_agg_first_item,
                  v->d_agg_item_sums, v->d_proj, v->d_item_sums};
  for (void* q : ptrs)
    if (q) (void)hipFree(q);
  v->d_row_segs = v->d_col_segs = nullptr;
  v->d_task_row_seg = v->d_task_col_seg = v->d_task_first_item = v->d_agg_first_item = nullptr;
  v->d_items = v->d_agg_items = nullptr;
  v->d_proj = v->d_item_sums = v->d_agg_item_sums = nullptr;
}

void free_subset_ring(cleave::SubsetRing* r) {
  if (r->d_ring) (void)hipFree(r->d_ring);
  if (r->d_captured) (void)hipFree(r->d_captured);
  for (const auto& f : r->in_flight) (void)hipEventDestroy(f.done);
  for (hipEvent_t e : r->idle_events) (void)hipEventDestroy(e);
  r->d_ring = r->d_captured = nullptr;
  r->in_flight.clear();
  r->idle_events.clear();
  r->max_items = r->pos = r->captured_used = 0;
}

void free_device_tables(cleave_plan* p) {
  free_verify_device(p->verify);
  if (p->d_tasks) (void)hipFree(p->d_tasks);
  for (int c = 0; c < cleave::kNumTileClasses; ++c)
    if (p->d_items[c]) (void)hipFree(p->d_items[c]);
  if (p->d_reduce_items) (void)hipFree(p->d_reduce_items);
  free_subset_ring(&p->subset);
  p->d_tasks = nullptr;
  if (p->d_items_fine) (void)hipFree(p->d_items_fine);
  p->d_items_fine = nullptr;
  for (int list = 0; list < cleave::kNumTileClasses + 1; ++list) {
    if (p->d_wg_ranges[list]) (void)hipFree(p->d_wg_ranges[list]);
    p->d_wg_ranges[list] = nullptr;
    p->wg_ranges_grid[list] = 0;
  }
  p->d_items[0] = p->d_items[1] = nullptr;
  p->d_reduce_items = nullptr;
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

// Work-list memory of cleave_execute_noalloc: a fixed array in the code
// object, one copy per GPU the library runs on, held until the process ends
// (768 KB).  In host code the name is only a handle for hipGetSymbolAddress;
// the address that kernels and copies use is g_static_scratch[device].
constexpr int64_t kStaticScratchItems = 16384;
static __device__ __align__(256) __attribute__((used))
unsigned char scratch[kStaticScratchItems * sizeof(cleave::WorkItem)];

// Once per device and process: the execute kernels' dynamic-LDS limits, the
// CU count and the address of this device's copy of `scratch`.  Done when a
// plan's tables are uploaded, so that no launch has to.
constexpr int kMaxDevices = 64;
std::mutex g_device_mu;
int g_device_cus[kMaxDevices] = {};   // 0 = not initialised
cleave::WorkItem* g_static_scratch[kMaxDevices] = {};

int ensure_device_ready(int dev, int* cus) {
  if (dev < 0 || dev >= kMaxDevices) return CLEAVE_EINVAL;
  std::lock_guard<std::mutex> lock(g_device_mu);
  if (g_device_cus[dev] == 0) {
    CLEAVE_HIP(cleave::configure_execute_kernels());
    CLEAVE_HIP(cleave::configure_execute_direct_kernels());
    void* ptr = nullptr;   // `dev` is the current device: its copy of the array
    CLEAVE_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    g_static_scratch[dev] = static_cast<cleave::WorkItem*>(ptr);
    int n = 0;
    CLEAVE_HIP(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
    g_device_cus[dev] = std::max(n, 1);
  }
  if (cus) *cus = g_device_cus[dev];
  return CLEAVE_OK;
}

constexpr int kSubsetEvents = 16;

int allocate_subset_ring(cleave_plan* p) {
  cleave::SubsetRing& r = p->subset;
  r.max_items = static_cast<int64_t>(std::max(p->items[0].size() + p->items[1].size(), p->items_fine.size()));
  if (r.max_items == 0) return CLEAVE_OK;
  const size_t item_bytes = static_cast<size_t>(r.max_items) * sizeof(cleave::WorkItem);
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&r.d_ring), 2 * item_bytes);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&r.d_captured), item_bytes);
  if (e == hipErrorOutOfMemory) return CLEAVE_ENOMEM;
  if (e != hipSuccess) return hip_fail(e);
  try {
    r.idle_events.reserve(kSubsetEvents);
    r.in_flight.reserve(kSubsetEvents);
  } catch (const std::bad_alloc&) {
    return CLEAVE_ENOMEM;
  }
  for (int i = 0; i < kSubsetEvents; ++i) {
    hipEvent_t ev = nullptr;
    CLEAVE_HIP(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
    r.idle_events.push_back(ev);
  }
  return CLEAVE_OK;
}

int ensure_uploaded(cleave_plan* p) {
  int dev = 0;
  CLEAVE_HIP(hipGetDevice(&dev));
  if (p->device == dev) return CLEAVE_OK;
  if (p->device >= 0) free_device_tables(p);
  int rc = ensure_device_ready(dev, nullptr);
  if (rc != CLEAVE_OK) return rc;
  rc = upload_vector(p->tasks, &p->d_tasks);
  // The three work-item lists; items of unequal length get a balanced workgroup
  // schedule for this device's grid (a copy is reordered: the host lists keep
  // their canonical order for the next device).
  int cus = 0;
  if (rc == CLEAVE_OK) rc = ensure_device_ready(dev, &cus);
  for (int list = 0; rc == CLEAVE_OK && list < cleave::kNumTileClasses + 1; ++list) {
    const bool fine = list == cleave::kNumTileClasses;
    const int cls = fine ? cleave::kTileSmall : list;
    const std::vector<cleave::WorkItem>& host = fine ? p->items_fine : p->items[list];
    const size_t n_direct = fine ? p->items_fine_whole_steps : p->items_whole_steps[list];
    cleave::WorkItem** dst = fine ? &p->d_items_fine : &p->d_items[list];
    const int64_t resident = static_cast<int64_t>(cus) * cleave::direct_workgroups_per_cu(cls);
    const int grid = static_cast<int>(std::min<int64_t>(static_cast<int64_t>(n_direct), resident));
    std::vector<uint32_t> ranges;
    try {
      std::vector<cleave::WorkItem> copy(host);
      cleave::balance_work_items(copy, n_direct, grid, &ranges);
      rc = upload_vector(ranges.empty() ? host : copy, dst);
    } catch (const std::bad_alloc&) {
      rc = CLEAVE_ENOMEM;
    }
    if (rc == CLEAVE_OK && !ranges.empty()) {
      rc = upload_vector(ranges, &p->d_wg_ranges[list]);
      p->wg_ranges_grid[list] = grid;
    }
  }
  if (rc == CLEAVE_OK) rc = upload_vector(p->reduce_items, &p->d_reduce_items);
  if (rc == CLEAVE_OK) rc = allocate_subset_ring(p);
  if (rc != CLEAVE_OK) {
    free_device_tables(p);
    return rc;
  }
  p->device = dev;
  return CLEAVE_OK;
}

int compute_units(int* out) {
  int dev = 0;
  CLEAVE_HIP(hipGetDevice(&dev));
  return ensure_device_ready(dev, out);
}

// A slice of `total` work items for a subset launch on `stream`.  Eager
// launches take the next slice of the ring (waiting, on the host, only for
// earlier launches that still read the slice: none unless the ring has
// wrapped onto unfinished work); launches under stream capture take a slice
// of the second buffer that is never handed out again.  No allocation.
int acquire_subset_slice(cleave::SubsetRing& r, int64_t total, bool capturing, cleave::WorkItem** out,
                         int64_t* begin) {
  if (total > r.max_items) return CLEAVE_EINVAL;   // cannot happen for distinct task ids
  if (capturing) {
    if (r.captured_used + total > r.max_items) return CLEAVE_ENOMEM;
    *out = r.d_captured + r.captured_used;
    *begin = -1;
    r.captured_used += total;
    return CLEAVE_OK;
  }
  if (r.pos + total > 2 * r.max_items) r.pos = 0;
  const int64_t b = r.pos, e = r.pos + total;
  // launches retire in order per stream, not across streams: check every record
  for (size_t i = 0; i < r.in_flight.size();) {
    const auto f = r.in_flight[i];
    const bool overlaps = f.begin < e && b < f.end;
    hipError_t q = overlaps ? hipEventSynchronize(f.done) : hipEventQuery(f.done);
    if (q == hipSuccess) {
      r.idle_events.push_back(f.done);
      r.in_flight.erase(r.in_flight.begin() + static_cast<std::ptrdiff_t>(i));
    } else if (q == hipErrorNotReady) {
      ++i;
    } else {
      return hip_fail(q);
    }
  }
  *out = r.d_ring + b;
  *begin = b;
  r.pos = e;
  return CLEAVE_OK;
}

// Marks the slice [begin, begin + total) as read by what has been enqueued on
// `stream` so far.
int release_subset_slice(cleave::SubsetRing& r, int64_t begin, int64_t total, hipStream_t stream) {
  if (begin < 0) return CLEAVE_OK;   // captured: never reused
  if (r.idle_events.empty()) {
    // every event is attached to a launch still in flight: wait for the oldest
    const auto f = r.in_flight.front();
    CLEAVE_HIP(hipEventSynchronize(f.done));
    r.in_flight.erase(r.in_flight.begin());
    r.idle_events.push_back(f.done);
  }
  hipEvent_t ev = r.idle_events.back();
  r.idle_events.pop_back();
  const hipError_t e = hipEventRecord(ev, stream);
  if (e != hipSuccess) {
    r.idle_events.push_back(ev);
    return hip_fail(e);
  }
  r.in_flight.push_back({begin, begin + total, ev});
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

extern "C" int cleave_version(void) { return 107; }

extern "C" int cleave_plan_upload(cleave_plan* plan) {
  if (!plan) return CLEAVE_EINVAL;
  return ensure_uploaded(plan);
}

extern "C" void cleave_plan_destroy(cleave_plan* plan) {
  if (!plan) return;
  if (plan->device >= 0) free_device_tables(plan);
  delete plan->verify;
  delete plan;
}

namespace {

// How a batched call finds its members' matrices (element offsets from the
// base pointers); all zero for a plain plan.
struct BatchLayout {
  cleave::BatchShape shape{0, 0};
  cleave::MemberOffsets a{}, b{};
  cleave::MemberOffsets c{};   // assemble mode and reduce only
};

// Every member offset is a multiple of `e` elements.
bool offsets_multiple_of(const cleave::MemberOffsets& at, const cleave::BatchShape& shape, int64_t e) {
  if (shape.n_group == 0) return at.outer % e == 0 && at.inner % e == 0;
  for (uint32_t g = 0; g < shape.n_group; ++g)
    if (at.table[g] % e != 0) return false;
  return true;
}

BatchLayout strided_layout(int64_t n_inner, int64_t a_outer, int64_t a_inner, int64_t b_outer,
                           int64_t b_inner, int64_t c_outer, int64_t c_inner) {
  BatchLayout bl;
  bl.shape.batch_inner = static_cast<uint32_t>(n_inner);
  bl.a.outer = a_outer;
  bl.a.inner = a_inner;
  bl.b.outer = b_outer;
  bl.b.inner = b_inner;
  bl.c.outer = c_outer;
  bl.c.inner = c_inner;
  return bl;
}

// Grouped launch: members given by one pointer each.  list[0] becomes the base
// pointer, the others element offsets from it.
int group_offsets(const void* const* list, int64_t n, int elem_bytes, cleave::MemberOffsets* at,
                  const void** base) {
  if (!list || n < 1 || n > cleave::kMaxGroup) return CLEAVE_EINVAL;
  for (int64_t g = 0; g < n; ++g)
    if (!list[g] || !aligned(list[g], elem_bytes)) return CLEAVE_EINVAL;
  *base = list[0];
  for (int64_t g = 0; g < n; ++g)
    at->table[g] = (reinterpret_cast<intptr_t>(list[g]) - reinterpret_cast<intptr_t>(list[0])) / elem_bytes;
  return CLEAVE_OK;
}

// Assemble mode: blocks go to their place in C instead of the partial buffer.
struct AssembleTarget {
  void* C = nullptr;
  int64_t ldc = 0;
  int out_dtype = CLEAVE_F32;
};

// Where the work items of a subset go: one list per tile class, each in two
// parts -- first the tasks whose chunk is a whole number of the direct
// kernel's K steps, then the others -- with the caller's order kept inside
// each part (the layout of the plan's own lists).
struct SubsetLayout {
  bool fine = false;                                  // every block cut into small-class sub-tiles
  int64_t counts[cleave::kNumTileClasses][2] = {};    // work items per (class, part)
  int64_t total() const { return counts[0][0] + counts[0][1] + counts[1][0] + counts[1][1]; }
};
inline int subset_part(const cleave_task& t) { return t.k_len % cleave::kDirectKStep == 0 ? 0 : 1; }

// Validates the ids (range, no repeats) and sizes the lists.  Uses the plan's
// own stamp array for the repeat check: no allocation.  Caller holds subset.mu.
int layout_subset(cleave_plan* plan, const int64_t* task_ids, int64_t n_ids, int cus, SubsetLayout* out) {
  const int64_t n_tasks = static_cast<int64_t>(plan->tasks.size());
  if (++plan->seen_generation == 0) {   // wrapped: start over with clean stamps
    std::fill(plan->seen_stamp.begin(), plan->seen_stamp.end(), 0u);
    plan->seen_generation = 1;
  }
  size_t large_items = 0;
  for (int64_t i = 0; i < n_ids; ++i) {
    const int64_t id = task_ids[i];
    if (id < 0 || id >= n_tasks || plan->seen_stamp[id] == plan->seen_generation) return CLEAVE_EINVAL;
    plan->seen_stamp[id] = plan->seen_generation;
    const cleave::SubTiling st = cleave::sub_tiling(plan->tasks[id], false);
    if (st.cls == cleave::kTileLarge) large_items += st.count();
  }
  // Few large items would leave most CUs idle: cut everything small instead
  // (the bits do not depend on the cut).
  out->fine = large_items > 0 && large_items <= static_cast<size_t>(cus) / 2;
  for (int64_t i = 0; i < n_ids; ++i) {
    const cleave_task& t = plan->tasks[task_ids[i]];
    const cleave::SubTiling st = cleave::sub_tiling(t, out->fine);
    out->counts[st.cls][subset_part(t)] += st.count();
  }
  return CLEAVE_OK;
}

// Enqueues the kernels that write the subset's work items to `out`; the
// (task, destination) pairs are built on the stack, one launch's worth at a time.
int expand_subset(const cleave_plan* plan, const int64_t* task_ids, int64_t n_ids,
                  const SubsetLayout& layout, cleave::WorkItem* out, hipStream_t stream) {
  int64_t next[cleave::kNumTileClasses][2];
  int64_t pos = 0;
  for (int c = 0; c < cleave::kNumTileClasses; ++c)
    for (int part = 0; part < 2; ++part) {
      next[c][part] = pos;
      pos += layout.counts[c][part];
    }
  cleave::ExpandArgs ea{};
  ea.tasks = plan->d_tasks;
  ea.out = out;
  ea.fine = layout.fine ? 1u : 0u;
  for (int64_t i = 0; i < n_ids; ++i) {
    const cleave_task& t = plan->tasks[task_ids[i]];
    const cleave::SubTiling st = cleave::sub_tiling(t, layout.fine);
    int64_t& at = next[st.cls][subset_part(t)];
    ea.entries[ea.n_entries++] = {static_cast<uint32_t>(task_ids[i]), static_cast<uint32_t>(at)};
    at += st.count();
    if (ea.n_entries == cleave::kSubsetEntriesPerLaunch || i + 1 == n_ids) {
      CLEAVE_HIP(cleave::launch_expand_subset(ea, stream));
      ea.n_entries = 0;
    }
  }
  return CLEAVE_OK;
}

int execute_impl(cleave_plan* plan, const int64_t* task_ids, int64_t n_ids, const void* A,
                 int64_t lda, int transA, const void* B, int64_t ldb, int transB, int dtype,
                 float* partials, const BatchLayout& bl, void* hip_stream,
                 const AssembleTarget& asm_to = AssembleTarget{}, bool static_scratch = false) {
  if (!plan || !A || !B || (!partials && !asm_to.C)) return CLEAVE_EINVAL;
  if (dtype != CLEAVE_F32 && dtype != CLEAVE_BF16) return CLEAVE_EINVAL;
  if ((transA != 0 && transA != 1) || (transB != 0 && transB != 1)) return CLEAVE_EINVAL;
  if ((task_ids == nullptr) != (n_ids == 0) || n_ids < 0) return CLEAVE_EINVAL;
  if (lda < (transA ? plan->M : plan->K) || ldb < (transB ? plan->K : plan->N)) return CLEAVE_EINVAL;
  const int eb = dtype == CLEAVE_BF16 ? 2 : 4;
  if (!aligned(A, eb) || !aligned(B, eb) || !aligned(partials, 4)) return CLEAVE_EINVAL;   // null partials: assemble mode
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);

  int cus = 0;
  int rc = compute_units(&cus);
  if (rc != CLEAVE_OK) return rc;
  // The large class runs one workgroup per CU; when its items would leave
  // half of the CUs or more idle, every block is cut into small sub-tiles
  // instead (four times as many items, two workgroups per CU).  The bits do
  // not depend on the cut.
  const auto prefers_fine = [cus](size_t large_items) {
    return large_items > 0 && large_items <= static_cast<size_t>(cus) / 2;
  };

  int dev = 0;
  CLEAVE_HIP(hipGetDevice(&dev));
  if (static_scratch) {
    // this entry point never allocates: the tables must be on the device already
    if (plan->device != dev) return CLEAVE_EINVAL;
  } else {
    rc = ensure_uploaded(plan);
    if (rc != CLEAVE_OK) return rc;
  }

  // 16-byte load path: every chunk and tile edge a multiple of 16 bytes and
  // all rows of both operands starting on 16-byte boundaries.
  const int e = 16 / eb;
  const bool vec = (e == 8 ? (plan->all_k_mult8 && plan->all_mn_mult8)
                           : (plan->all_k_mult4 && plan->all_mn_mult4)) &&
                   lda % e == 0 && ldb % e == 0 && aligned(A, 16) && aligned(B, 16) &&
                   // in-tile byte offsets are kept in 32 bits
                   lda * eb < (int64_t{1} << 22) && ldb * eb < (int64_t{1} << 22) &&
                   offsets_multiple_of(bl.a, bl.shape, e) && offsets_multiple_of(bl.b, bl.shape, e);

  const cleave::WorkItem* d_lists[cleave::kNumTileClasses] = {plan->d_items[0], plan->d_items[1]};
  int64_t counts[cleave::kNumTileClasses] = {static_cast<int64_t>(plan->items[0].size()),
                                             static_cast<int64_t>(plan->items[1].size())};
  // leading items of each list whose chunk is a whole number of direct-kernel K steps
  int64_t whole_steps[cleave::kNumTileClasses] = {static_cast<int64_t>(plan->items_whole_steps[0]),
                                                  static_cast<int64_t>(plan->items_whole_steps[1])};
  // which of the plan's lists a class runs from (-1: a subset's own list)
  int list_of[cleave::kNumTileClasses] = {task_ids ? -1 : 0, task_ids ? -1 : 1};
  if (!task_ids && prefers_fine(plan->items[cleave::kTileLarge].size())) {
    list_of[cleave::kTileSmall] = cleave::kNumTileClasses;
    d_lists[cleave::kTileLarge] = nullptr;
    counts[cleave::kTileLarge] = 0;
    whole_steps[cleave::kTileLarge] = 0;
    d_lists[cleave::kTileSmall] = plan->d_items_fine;
    counts[cleave::kTileSmall] = static_cast<int64_t>(plan->items_fine.size());
    whole_steps[cleave::kTileSmall] = static_cast<int64_t>(plan->items_fine_whole_steps);
  }
  // Subset launches: the work-item lists are written on the device, from the
  // task records, into a slice of memory the plan set aside when its tables
  // were uploaded -- stream-ordered, no host wait, no copy, no allocation.
  std::unique_lock<std::mutex> subset_lock;
  int64_t slice_begin = -1, slice_total = 0;
  if (task_ids) {
    subset_lock = std::unique_lock<std::mutex>(plan->subset.mu);
    SubsetLayout layout;
    rc = layout_subset(plan, task_ids, n_ids, cus, &layout);
    if (rc != CLEAVE_OK) return rc;
    slice_total = layout.total();
    cleave::WorkItem* slice = nullptr;
    if (static_scratch) {
      // the device's fixed array, from its start: whatever an earlier call left there is overwritten
      if (slice_total > kStaticScratchItems) return CLEAVE_ELIMIT;
      slice = g_static_scratch[dev];
    } else {
      hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
      CLEAVE_HIP(hipStreamIsCapturing(stream, &capture));
      rc = acquire_subset_slice(plan->subset, slice_total, capture != hipStreamCaptureStatusNone, &slice,
                                &slice_begin);
      if (rc != CLEAVE_OK) return rc;
    }
    rc = expand_subset(plan, task_ids, n_ids, layout, slice, stream);
    if (rc != CLEAVE_OK) {
      if (!static_scratch) (void)release_subset_slice(plan->subset, slice_begin, slice_total, stream);
      return rc;
    }
    int64_t pos = 0;
    for (int c = 0; c < cleave::kNumTileClasses; ++c) {
      d_lists[c] = slice + pos;
      whole_steps[c] = layout.counts[c][0];
      counts[c] = layout.counts[c][0] + layout.counts[c][1];
      pos += counts[c];
    }
  }

  // whatever has been enqueued reads the slice: mark it even if a later launch fails
  const auto launch_failed = [&](hipError_t e) {
    if (task_ids && !static_scratch) (void)release_subset_slice(plan->subset, slice_begin, slice_total, stream);
    return hip_fail(e);
  };
  int64_t most = -1;
  for (int c = 0; c < cleave::kNumTileClasses; ++c) {
    if (counts[c] == 0) continue;
    cleave::ExecuteArgs args{};
    args.items = d_lists[c];
    args.n_items = counts[c];
    args.A = A;
    args.B = B;
    args.lda = lda;
    args.ldb = ldb;
    args.transA = transA;
    args.transB = transB;
    args.partials = partials;
    args.batch = bl.shape;
    args.a_at = bl.a;
    args.b_at = bl.b;
    args.c_at = bl.c;
    args.C = asm_to.C;
    args.ldc = asm_to.ldc;
    args.c_bf16 = asm_to.out_dtype == CLEAVE_BF16 ? 1 : 0;
    // block origins and row lengths are multiples of 8 elements whenever `vec` holds
    args.out_vec = !vec ? 0
                   : !asm_to.C ? aligned(partials, 16)
                               : (asm_to.ldc % 4 == 0 && aligned(asm_to.C, args.c_bf16 ? 8 : 16) &&
                                  offsets_multiple_of(bl.c, bl.shape, 4));
    // bf16 with 16-byte loads: items made of whole K steps go to the direct
    // kernel, the others (if any) to the staged one.  Which kernel computes a
    // block depends only on the block's own task record.
    const int64_t n_direct = (vec && dtype == CLEAVE_BF16) ? whole_steps[c] : 0;
    const int64_t n_staged = counts[c] - n_direct;
    if (n_direct > 0) {
      // Persistent workgroups, as many as the chip holds at once: each walks
      // the item list with the grid as stride and fetches the head of its next
      // item while it stores the current one.
      args.items = d_lists[c];
      args.n_items = n_direct;
      const int64_t resident = static_cast<int64_t>(cus) * cleave::direct_workgroups_per_cu(c);
      const int grid = static_cast<int>(std::min<int64_t>(n_direct, resident));
      // items of unequal length: the schedule made for this grid when the tables were uploaded
      const int list = list_of[c];
      args.wg_ranges = (list >= 0 && plan->wg_ranges_grid[list] == grid) ? plan->d_wg_ranges[list] : nullptr;
      const hipError_t he = cleave::launch_execute_direct(args, c, grid, stream);
      args.wg_ranges = nullptr;
      if (he != hipSuccess) return launch_failed(he);
    }
    if (n_staged > 0) {
      // One workgroup per work item (the kernel loops only if the grid is
      // capped): the hardware dispatcher then balances uneven items and keeps
      // the workgroups that share a CU out of phase.
      args.items = d_lists[c] + n_direct;
      args.n_items = n_staged;
      constexpr int64_t kMaxGrid = int64_t{1} << 20;
      const int grid = static_cast<int>(std::min<int64_t>(n_staged, kMaxGrid));
      const hipError_t he = cleave::launch_execute(args, dtype, c, vec, grid, stream);
      if (he != hipSuccess) return launch_failed(he);
    }
    if (counts[c] > most) {
      most = counts[c];
      plan->last_kernel = n_direct >= n_staged ? direct_kernel_name(c, transA, transB)
                                               : kernel_name(dtype, c, vec, transA, transB);
    }
  }
  if (task_ids && !static_scratch) return release_subset_slice(plan->subset, slice_begin, slice_total, stream);
  return CLEAVE_OK;
}

}  // namespace

extern "C" int cleave_execute(cleave_plan* plan, const int64_t* task_ids, int64_t n_ids,
                              const void* A, int64_t lda, int transA, const void* B, int64_t ldb,
                              int transB, int dtype, float* partials, void* hip_stream) {
  if (plan && plan->batch > 0) return CLEAVE_EINVAL;   // batched plans use the batched call
  return execute_impl(plan, task_ids, n_ids, A, lda, transA, B, ldb, transB, dtype, partials,
                      BatchLayout{}, hip_stream);
}

extern "C" int cleave_execute_noalloc(cleave_plan* plan, const int64_t* task_ids, int64_t n_ids,
                                      const void* A, int64_t lda, int transA, const void* B,
                                      int64_t ldb, int transB, int dtype, float* partials,
                                      void* hip_stream) {
  if (plan && plan->batch > 0) return CLEAVE_EINVAL;
  return execute_impl(plan, task_ids, n_ids, A, lda, transA, B, ldb, transB, dtype, partials,
                      BatchLayout{}, hip_stream, AssembleTarget{}, true);
}

extern "C" int cleave_execute_batched(cleave_plan* plan, const int64_t* task_ids, int64_t n_ids,
                                      const void* A, int64_t lda, int transA, int64_t a_outer,
                                      int64_t a_inner, const void* B, int64_t ldb, int transB,
                                      int64_t b_outer, int64_t b_inner, int64_t n_inner, int dtype,
                                      float* partials, void* hip_stream) {
  if (!plan || plan->batch < 1) return CLEAVE_EINVAL;
  if (n_inner < 1 || n_inner > std::numeric_limits<uint32_t>::max() || plan->batch % n_inner != 0)
    return CLEAVE_EINVAL;
  if (a_outer < 0 || a_inner < 0 || b_outer < 0 || b_inner < 0) return CLEAVE_EINVAL;
  return execute_impl(plan, task_ids, n_ids, A, lda, transA, B, ldb, transB, dtype, partials,
                      strided_layout(n_inner, a_outer, a_inner, b_outer, b_inner, 0, 0), hip_stream);
}

extern "C" int cleave_execute_grouped(cleave_plan* plan, const int64_t* task_ids, int64_t n_ids,
                                      int64_t n_members, const void* const* A_list, int64_t lda,
                                      int transA,
                                      const void* const* B_list, int64_t ldb, int transB, int dtype,
                                      float* partials, void* hip_stream) {
  if (!plan || plan->batch < 1 || plan->batch > cleave::kMaxGroup || n_members != plan->batch)
    return CLEAVE_EINVAL;
  if (dtype != CLEAVE_F32 && dtype != CLEAVE_BF16) return CLEAVE_EINVAL;
  const int eb = dtype == CLEAVE_BF16 ? 2 : 4;
  BatchLayout bl;
  bl.shape.n_group = static_cast<uint32_t>(plan->batch);
  const void* A = nullptr;
  const void* B = nullptr;
  int rc = group_offsets(A_list, plan->batch, eb, &bl.a, &A);
  if (rc != CLEAVE_OK) return rc;
  rc = group_offsets(B_list, plan->batch, eb, &bl.b, &B);
  if (rc != CLEAVE_OK) return rc;
  return execute_impl(plan, task_ids, n_ids, A, lda, transA, B, ldb, transB, dtype, partials, bl,
                      hip_stream);
}

extern "C" int cleave_execute_assemble(cleave_plan* plan, const int64_t* task_ids, int64_t n_ids,
                                       const void* A, int64_t lda, int transA, int64_t a_outer,
                                       int64_t a_inner, const void* B, int64_t ldb, int transB,
                                       int64_t b_outer, int64_t b_inner, int64_t n_inner, int dtype,
                                       void* C, int64_t ldc, int64_t c_outer, int64_t c_inner,
                                       int out_dtype, void* hip_stream) {
  if (!plan || !C) return CLEAVE_EINVAL;
  if (out_dtype != CLEAVE_F32 && out_dtype != CLEAVE_BF16) return CLEAVE_EINVAL;
  if (ldc < plan->N || !aligned(C, out_dtype == CLEAVE_BF16 ? 2 : 4)) return CLEAVE_EINVAL;
  // a block is the finished output only if its task covers the whole inner dimension
  for (const cleave_task& t : plan->tasks)
    if (t.ksplit_cnt != 1) return CLEAVE_EINVAL;
  BatchLayout bl;
  if (plan->batch > 0) {
    if (n_inner < 1 || n_inner > std::numeric_limits<uint32_t>::max() || plan->batch % n_inner != 0)
      return CLEAVE_EINVAL;
    if (a_outer < 0 || a_inner < 0 || b_outer < 0 || b_inner < 0 || c_outer < 0 || c_inner < 0)
      return CLEAVE_EINVAL;
    bl = strided_layout(n_inner, a_outer, a_inner, b_outer, b_inner, c_outer, c_inner);
  } else if (n_inner != 0 || a_outer || a_inner || b_outer || b_inner || c_outer || c_inner) {
    return CLEAVE_EINVAL;   // strides belong to batched plans
  }
  AssembleTarget to;
  to.C = C;
  to.ldc = ldc;
  to.out_dtype = out_dtype;
  return execute_impl(plan, task_ids, n_ids, A, lda, transA, B, ldb, transB, dtype, nullptr, bl,
                      hip_stream, to);
}

namespace {

// Which operator consumes the aggregated values.
struct ReduceEpilogue {
  const void* residual = nullptr;          // C = sum + residual
  const cleave::AdamArgs* adam = nullptr;  // Adam update of adam->w (C unused)
  const cleave::AdamGroupOffsets* adam_group = nullptr;   // with adam: one set of arrays per member
};

int reduce_impl(cleave_plan* plan, const float* partials, void* C, int64_t ldc, int out_dtype,
                const BatchLayout& bl, void* hip_stream,
                const ReduceEpilogue& epi = ReduceEpilogue{}, bool members_aligned = true) {
  if (!plan || !partials || !C) return CLEAVE_EINVAL;
  if (out_dtype != CLEAVE_F32 && out_dtype != CLEAVE_BF16) return CLEAVE_EINVAL;
  if (ldc < plan->N) return CLEAVE_EINVAL;
  const int ob = out_dtype == CLEAVE_BF16 ? 2 : 4;
  if (!aligned(partials, 4) || !aligned(C, ob)) return CLEAVE_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);

  int rc = ensure_uploaded(plan);
  if (rc != CLEAVE_OK) return rc;

  bool vec = plan->all_n_mult4 && ldc % 4 == 0 && aligned(partials, 16) && aligned(C, 4 * ob) &&
             offsets_multiple_of(bl.c, bl.shape, 4) && members_aligned;
  if (epi.residual) vec = vec && aligned(epi.residual, 4 * ob);
  if (epi.adam)
    vec = vec && aligned(epi.adam->m, 16) && aligned(epi.adam->v, 16) &&
          (!epi.adam->w_bf16 || aligned(epi.adam->w_bf16, 8));
  cleave::ReduceArgs args{};
  args.tasks = plan->d_tasks;
  args.items = plan->d_reduce_items;
  args.n_items = static_cast<int64_t>(plan->reduce_items.size());
  args.partials = partials;
  args.C = C;
  args.ldc = ldc;
  args.batch = bl.shape;
  args.c_at = bl.c;
  // one workgroup per reduce item (the kernel loops only if the grid is capped)
  const int grid = static_cast<int>(std::min<int64_t>(args.n_items, int64_t{1} << 20));
  if (epi.adam && epi.adam_group) {
    CLEAVE_HIP(cleave::launch_reduce_adam_grouped(args, *epi.adam, *epi.adam_group, vec, grid, stream));
  } else if (epi.adam) {
    CLEAVE_HIP(cleave::launch_reduce_adam(args, *epi.adam, vec, grid, stream));
  } else if (epi.residual) {
    CLEAVE_HIP(cleave::launch_reduce_residual(args, epi.residual, out_dtype, vec, grid, stream));
  } else {
    CLEAVE_HIP(cleave::launch_reduce(args, out_dtype, vec, grid, stream));
  }
  return CLEAVE_OK;
}

}  // namespace

extern "C" int cleave_reduce_residual(cleave_plan* plan, const float* partials, const void* R,
                                      void* C, int64_t ldc, int out_dtype, void* hip_stream) {
  if (!R || (plan && plan->batch > 0)) return CLEAVE_EINVAL;
  if (out_dtype != CLEAVE_F32 && out_dtype != CLEAVE_BF16) return CLEAVE_EINVAL;
  if (!aligned(R, out_dtype == CLEAVE_BF16 ? 2 : 4)) return CLEAVE_EINVAL;
  ReduceEpilogue epi;
  epi.residual = R;
  return reduce_impl(plan, partials, C, ldc, out_dtype, BatchLayout{}, hip_stream, epi);
}

extern "C" int cleave_reduce_adam(cleave_plan* plan, const float* partials, float* w, float* m,
                                  float* v, void* w_bf16, int64_t ld, float lr, float beta1,
                                  float beta2, float eps, float weight_decay, int64_t step,
                                  void* hip_stream) {
  if (!w || !m || !v || (plan && plan->batch > 0)) return CLEAVE_EINVAL;
  if (step < 1 || !(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f) ||
      !(eps >= 0.0f) || !(lr == lr) || !(weight_decay == weight_decay))
    return CLEAVE_EINVAL;
  if (!aligned(m, 4) || !aligned(v, 4) || !aligned(w_bf16, 2)) return CLEAVE_EINVAL;
  cleave::AdamArgs h{};
  h.w = w;
  h.m = m;
  h.v = v;
  h.w_bf16 = static_cast<uint16_t*>(w_bf16);
  h.lr = lr;
  h.beta1 = beta1;
  h.beta2 = beta2;
  h.eps = eps;
  h.weight_decay = weight_decay;
  h.inv_bias1 = static_cast<float>(1.0 / (1.0 - std::pow(static_cast<double>(beta1), static_cast<double>(step))));
  h.inv_bias2 = static_cast<float>(1.0 / (1.0 - std::pow(static_cast<double>(beta2), static_cast<double>(step))));
  ReduceEpilogue epi;
  epi.adam = &h;
  // the fp32 master weight takes C's place in the common checks (pointer, leading dimension)
  return reduce_impl(plan, partials, w, ld, CLEAVE_F32, BatchLayout{}, hip_stream, epi);
}

extern "C" int cleave_reduce_adam_grouped(cleave_plan* plan, const float* partials, int64_t n_members,
                                          float* const* w_list, float* const* m_list,
                                          float* const* v_list, void* const* w_bf16_list, int64_t ld,
                                          float lr, float beta1, float beta2, float eps,
                                          float weight_decay, int64_t step, void* hip_stream) {
  if (!plan || plan->batch < 1 || plan->batch > cleave::kMaxGroup || n_members != plan->batch)
    return CLEAVE_EINVAL;
  if (!w_list || !m_list || !v_list) return CLEAVE_EINVAL;
  if (step < 1 || !(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f) ||
      !(eps >= 0.0f) || !(lr == lr) || !(weight_decay == weight_decay))
    return CLEAVE_EINVAL;
  cleave::AdamGroupOffsets at{};
  bool all16 = true;
  for (int64_t g = 0; g < n_members; ++g) {
    if (!w_list[g] || !m_list[g] || !v_list[g] || (w_bf16_list && !w_bf16_list[g])) return CLEAVE_EINVAL;
    if (!aligned(w_list[g], 4) || !aligned(m_list[g], 4) || !aligned(v_list[g], 4) ||
        (w_bf16_list && !aligned(w_bf16_list[g], 2)))
      return CLEAVE_EINVAL;
    all16 = all16 && aligned(w_list[g], 16) && aligned(m_list[g], 16) && aligned(v_list[g], 16) &&
            (!w_bf16_list || aligned(w_bf16_list[g], 8));
    at.w[g] = w_list[g] - w_list[0];
    at.m[g] = m_list[g] - m_list[0];
    at.v[g] = v_list[g] - v_list[0];
    at.w_bf16[g] = w_bf16_list ? static_cast<uint16_t*>(w_bf16_list[g]) - static_cast<uint16_t*>(w_bf16_list[0]) : 0;
  }
  cleave::AdamArgs h{};
  h.w = w_list[0];
  h.m = m_list[0];
  h.v = v_list[0];
  h.w_bf16 = w_bf16_list ? static_cast<uint16_t*>(w_bf16_list[0]) : nullptr;
  h.lr = lr;
  h.beta1 = beta1;
  h.beta2 = beta2;
  h.eps = eps;
  h.weight_decay = weight_decay;
  h.inv_bias1 = static_cast<float>(1.0 / (1.0 - std::pow(static_cast<double>(beta1), static_cast<double>(step))));
  h.inv_bias2 = static_cast<float>(1.0 / (1.0 - std::pow(static_cast<double>(beta2), static_cast<double>(step))));
  ReduceEpilogue epi;
  epi.adam = &h;
  epi.adam_group = &at;
  BatchLayout bl;
  bl.shape.n_group = static_cast<uint32_t>(plan->batch);   // c_at stays zero: every array has its own table
  // reduce_impl's vector-path test looks at h's (member 0's) arrays; the members must agree
  // (a member whose arrays are not 16-byte aligned sends the whole launch down the element path)
  return reduce_impl(plan, partials, h.w, ld, CLEAVE_F32, bl, hip_stream, epi, all16);
}

extern "C" int cleave_reduce(cleave_plan* plan, const float* partials, void* C, int64_t ldc,
                             int out_dtype, void* hip_stream) {
  if (plan && plan->batch > 0) return CLEAVE_EINVAL;
  return reduce_impl(plan, partials, C, ldc, out_dtype, BatchLayout{}, hip_stream);
}

extern "C" int cleave_reduce_batched(cleave_plan* plan, const float* partials, void* C, int64_t ldc,
                                     int64_t c_outer, int64_t c_inner, int64_t n_inner,
                                     int out_dtype, void* hip_stream) {
  if (!plan || plan->batch < 1) return CLEAVE_EINVAL;
  if (n_inner < 1 || n_inner > std::numeric_limits<uint32_t>::max() || plan->batch % n_inner != 0)
    return CLEAVE_EINVAL;
  if (c_outer < 0 || c_inner < 0) return CLEAVE_EINVAL;
  return reduce_impl(plan, partials, C, ldc, out_dtype,
                     strided_layout(n_inner, 0, 0, 0, 0, c_outer, c_inner), hip_stream);
}

extern "C" int cleave_reduce_grouped(cleave_plan* plan, const float* partials, int64_t n_members,
                                     void* const* C_list, int64_t ldc, int out_dtype,
                                     void* hip_stream) {
  if (!plan || plan->batch < 1 || plan->batch > cleave::kMaxGroup || n_members != plan->batch)
    return CLEAVE_EINVAL;
  if (out_dtype != CLEAVE_F32 && out_dtype != CLEAVE_BF16) return CLEAVE_EINVAL;
  BatchLayout bl;
  bl.shape.n_group = static_cast<uint32_t>(plan->batch);
  const void* C = nullptr;
  const int rc = group_offsets(C_list, plan->batch, out_dtype == CLEAVE_BF16 ? 2 : 4, &bl.c, &C);
  if (rc != CLEAVE_OK) return rc;
  return reduce_impl(plan, partials, const_cast<void*>(C), ldc, out_dtype, bl, hip_stream);
}

#ifndef CLEAVE_AGG_ELEMS
#define CLEAVE_AGG_ELEMS 8192
#endif

namespace {

// Host tables of the returned-block check (built once per plan) and their
// device copies plus scratch (once per device the plan is used on).
int ensure_verify_tables_host(cleave_plan* p) {
  using cleave::Segment;
  using cleave::VerifyItem;
  if (!p->verify) {
    cleave::VerifyTables* v = new (std::nothrow) cleave::VerifyTables;
    if (!v) return CLEAVE_ENOMEM;
    try {
      std::map<std::pair<uint32_t, uint32_t>, uint32_t> rows, cols;
      // Elements of a partial block per bilinear item: long runs stream best
      // (measured +11 % with 8 splits of 4 MiB blocks), as long as the launch
      // still has a few thousand items to spread over the chip.
      const uint32_t kElemsPerItem = p->partial_elems >= (int64_t{2048} << 15) ? 32768u : 16384u;
      v->task_first_item.push_back(0);
      for (const cleave_task& t : p->tasks) {
        auto ri = rows.emplace(std::make_pair(t.m0, t.m_len), static_cast<uint32_t>(rows.size()));
        if (ri.second) v->row_segs.push_back(Segment{t.m0, t.m_len});
        v->task_row_seg.push_back(ri.first->second);
        auto ci = cols.emplace(std::make_pair(t.n0, t.n_len), static_cast<uint32_t>(cols.size()));
        if (ci.second) v->col_segs.push_back(Segment{t.n0, t.n_len});
        v->task_col_seg.push_back(ci.first->second);
        const uint32_t rows_per = std::max<uint32_t>(1, kElemsPerItem / t.n_len);
        const uint32_t index = static_cast<uint32_t>(&t - p->tasks.data());
        for (uint32_t r0 = 0; r0 < t.m_len; r0 += rows_per)
          v->items.push_back(VerifyItem{index, r0, std::min(rows_per, t.m_len - r0), 0});
        v->max_ksplit = std::max(v->max_ksplit, t.ksplit_cnt);
        if (v->items.size() > std::numeric_limits<uint32_t>::max()) {
          delete v;
          return CLEAVE_EINVAL;
        }
        v->task_first_item.push_back(static_cast<uint32_t>(v->items.size()));
      }
      for (const std::vector<Segment>* segs : {&v->row_segs, &v->col_segs})
        for (const Segment& sg : *segs) {
          v->segs_mult8 &= ((sg.start | sg.len) % 8 == 0);
          v->segs_mult4 &= ((sg.start | sg.len) % 4 == 0);
        }
    } catch (const std::bad_alloc&) {
      delete v;
      return CLEAVE_ENOMEM;
    }
    p->verify = v;
  }
  return CLEAVE_OK;
}

int ensure_verify_tables(cleave_plan* p) {
  int rc = ensure_verify_tables_host(p);
  if (rc != CLEAVE_OK) return rc;
  cleave::VerifyTables* v = p->verify;
  if (v->d_items || p->tasks.empty()) return CLEAVE_OK;
  rc = upload_vector(v->row_segs, &v->d_row_segs);
  if (rc == CLEAVE_OK) rc = upload_vector(v->col_segs, &v->d_col_segs);
  if (rc == CLEAVE_OK) rc = upload_vector(v->task_row_seg, &v->d_task_row_seg);
  if (rc == CLEAVE_OK) rc = upload_vector(v->task_col_seg, &v->d_task_col_seg);
  if (rc == CLEAVE_OK) rc = upload_vector(v->task_first_item, &v->d_task_first_item);
  if (rc == CLEAVE_OK) rc = upload_vector(v->items, &v->d_items);
  if (rc == CLEAVE_OK) {
    const size_t members = p->batch > 0 ? static_cast<size_t>(p->batch) : 1;
    const size_t proj = 2 * (v->row_segs.size() + v->col_segs.size()) * static_cast<size_t>(p->K) * members;
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&v->d_proj), proj * sizeof(double));
    if (e == hipSuccess)
      e = hipMalloc(reinterpret_cast<void**>(&v->d_item_sums), v->items.size() * sizeof(double));
    if (e == hipErrorOutOfMemory) rc = CLEAVE_ENOMEM;
    else if (e != hipSuccess) rc = hip_fail(e);
  }
  if (rc != CLEAVE_OK) free_verify_device(v);
  return rc;
}

// Tables of the fused check + aggregation (first fused call on the plan, after
// ensure_verify_tables): runs of rows of ~kAggElemsPerItem output elements.
int ensure_aggregate_tables(cleave_plan* p) {
  using cleave::VerifyItem;
  cleave::VerifyTables* v = p->verify;
  if (v->d_agg_items || p->tasks.empty()) return CLEAVE_OK;
  if (v->agg_first_item.empty()) {
    try {
      constexpr uint32_t kAggElemsPerItem = CLEAVE_AGG_ELEMS;
      uint64_t slots = 0;
      v->agg_first_item.push_back(0);
      for (const cleave_task& t : p->tasks) {
        const uint32_t rows_per = std::max<uint32_t>(1, kAggElemsPerItem / t.n_len);
        const uint32_t index = static_cast<uint32_t>(&t - p->tasks.data());
        for (uint32_t r0 = 0, j = 0; r0 < t.m_len; r0 += rows_per, ++j) {
          if (t.ksplit_idx == 0)
            v->agg_items.push_back(VerifyItem{index, r0, std::min(rows_per, t.m_len - r0),
                                              static_cast<uint32_t>(slots) + j});
        }
        slots += (t.m_len + rows_per - 1) / rows_per;
        if (slots > std::numeric_limits<uint32_t>::max()) {
          v->agg_items.clear();
          v->agg_first_item.clear();
          return CLEAVE_EINVAL;
        }
        v->agg_first_item.push_back(static_cast<uint32_t>(slots));
      }
    } catch (const std::bad_alloc&) {
      v->agg_items.clear();
      v->agg_first_item.clear();
      return CLEAVE_ENOMEM;
    }
  }
  int rc = upload_vector(v->agg_items, &v->d_agg_items);
  if (rc == CLEAVE_OK) rc = upload_vector(v->agg_first_item, &v->d_agg_first_item);
  if (rc == CLEAVE_OK) {
    const hipError_t e = hipMalloc(reinterpret_cast<void**>(&v->d_agg_item_sums),
                                   static_cast<size_t>(v->agg_first_item.back()) * sizeof(double));
    if (e == hipErrorOutOfMemory) rc = CLEAVE_ENOMEM;
    else if (e != hipSuccess) rc = hip_fail(e);
  }
  if (rc != CLEAVE_OK) {
    for (void* q : {static_cast<void*>(v->d_agg_items), static_cast<void*>(v->d_agg_first_item),
                    static_cast<void*>(v->d_agg_item_sums)})
      if (q) (void)hipFree(q);
    v->d_agg_items = nullptr;
    v->d_agg_first_item = nullptr;
    v->d_agg_item_sums = nullptr;
  }
  return rc;
}

}  // namespace

namespace {

// Where the fused pass writes the aggregated output (C == nullptr: check only).
struct AggregateTarget {
  void* C = nullptr;
  int64_t ldc = 0;
  int out_dtype = CLEAVE_F32;
};

int verify_impl(cleave_plan* plan, const void* A, int64_t lda, int transA, const void* B, int64_t ldb,
                int transB, int dtype, const float* partials, const float* r, const float* s, double tol,
                double* lhs, double* rhs, double* scale, int32_t* accept, const BatchLayout& bl,
                void* hip_stream, const AggregateTarget& agg = AggregateTarget{}) {
  if (!plan || !A || !B || !partials || !r || !s || !accept) return CLEAVE_EINVAL;
  if (dtype != CLEAVE_F32 && dtype != CLEAVE_BF16) return CLEAVE_EINVAL;
  if ((transA != 0 && transA != 1) || (transB != 0 && transB != 1)) return CLEAVE_EINVAL;
  if (lda < (transA ? plan->M : plan->K) || ldb < (transB ? plan->K : plan->N)) return CLEAVE_EINVAL;
  if (!(tol >= 0.0)) return CLEAVE_EINVAL;   // also refuses NaN
  const int eb = dtype == CLEAVE_BF16 ? 2 : 4;
  if (!aligned(A, eb) || !aligned(B, eb) || !aligned(partials, 4) || !aligned(r, 4) ||
      !aligned(s, 4) || !aligned(accept, 4) || !aligned(lhs, 8) || !aligned(rhs, 8) ||
      !aligned(scale, 8))
    return CLEAVE_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);

  int rc = ensure_uploaded(plan);
  if (rc != CLEAVE_OK) return rc;
  rc = ensure_verify_tables(plan);
  if (rc != CLEAVE_OK) return rc;
  cleave::VerifyTables* v = plan->verify;
  if (plan->tasks.empty()) return CLEAVE_OK;

  const int64_t K = plan->K;
  const bool batched = plan->batch > 0;
  const int n_members = batched ? static_cast<int>(plan->batch) : 1;
  const int e = 16 / eb;   // elements per 16-byte load
  const bool segs_ok = e == 8 ? v->segs_mult8 : v->segs_mult4;
  const size_t row_proj = v->row_segs.size() * static_cast<size_t>(K) * static_cast<size_t>(n_members);
  const size_t col_proj = v->col_segs.size() * static_cast<size_t>(K) * static_cast<size_t>(n_members);
  double* U = v->d_proj;
  double* U_abs = U + row_proj;
  double* V = U_abs + row_proj;
  double* V_abs = V + col_proj;

  // op(A)[i][k]: stored M x K (transA = 0) -> the summed row index strides;
  // stored K x M (transA = 1) -> it is contiguous.  op(B)[k][j]: stored K x N
  // (transB = 0) -> the summed column index is contiguous; stored N x K -> it
  // strides.
  const bool a_contig = transA != 0;
  const bool b_contig = transB == 0;
  // members' probe vectors follow each other: r is n_members x M, s is n_members x N
  const int64_t r_stride = batched ? plan->M : 0, s_stride = batched ? plan->N : 0;
  const bool a_vec = aligned(A, 16) && lda % e == 0 && offsets_multiple_of(bl.a, bl.shape, e) &&
                     (a_contig ? (segs_ok && aligned(r, 16) && r_stride % 4 == 0) : K % e == 0);
  const bool b_vec = aligned(B, 16) && ldb % e == 0 && offsets_multiple_of(bl.b, bl.shape, e) &&
                     (b_contig ? (segs_ok && aligned(s, 16) && s_stride % 4 == 0) : K % e == 0);
  const bool p_vec = plan->all_n_mult4 && aligned(partials, 16) && aligned(s, 16) && s_stride % 4 == 0;
  cleave::VerifyPassArgs pass{};
  pass.A = cleave::ProjectArgs{A, lda, v->d_row_segs, static_cast<int>(v->row_segs.size()), r, U, U_abs, K,
                               n_members, r_stride, bl.shape, bl.a};
  pass.B = cleave::ProjectArgs{B, ldb, v->d_col_segs, static_cast<int>(v->col_segs.size()), s, V, V_abs, K,
                               n_members, s_stride, bl.shape, bl.b};
  pass.bil = cleave::BilinearArgs{plan->d_tasks, v->d_items, static_cast<int64_t>(v->items.size()),
                                  partials, r, s, v->d_item_sums, batched ? 1 : 0, r_stride, s_stride};
  const uint32_t* first_item = v->d_task_first_item;
  const double* item_sums = v->d_item_sums;
  if (agg.C) {
    rc = ensure_aggregate_tables(plan);
    if (rc != CLEAVE_OK) return rc;
    first_item = v->d_agg_first_item;
    item_sums = v->d_agg_item_sums;
    const int ob = agg.out_dtype == CLEAVE_BF16 ? 2 : 4;
    const bool c_vec = agg.ldc % 4 == 0 && aligned(agg.C, 4 * ob);
    cleave::VerifyReducePassArgs fused{};
    fused.A = pass.A;
    fused.B = pass.B;
    fused.bil = pass.bil;
    fused.bil.item_sums = v->d_agg_item_sums;
    fused.agg = cleave::AggregateArgs{v->d_agg_items, static_cast<int64_t>(v->agg_items.size()),
                                      v->d_agg_first_item, agg.C, agg.ldc, agg.out_dtype == CLEAVE_BF16 ? 1 : 0};
    CLEAVE_HIP(cleave::launch_verify_reduce_pass(fused, dtype, a_contig, b_contig,
                                                 a_vec && b_vec && p_vec && c_vec, stream));
  } else {
    CLEAVE_HIP(cleave::launch_verify_pass(pass, dtype, a_contig, b_contig, a_vec && b_vec && p_vec, stream));
  }

  cleave::VerdictArgs va{plan->d_tasks, static_cast<int64_t>(plan->tasks.size()),
                         v->d_task_row_seg, v->d_task_col_seg, first_item,
                         item_sums, U, U_abs, V, V_abs, K, batched ? 1 : 0,
                         static_cast<int>(v->row_segs.size()), static_cast<int>(v->col_segs.size()),
                         tol, lhs, rhs, scale, accept};
  CLEAVE_HIP(cleave::launch_verdict(va, stream));
  return CLEAVE_OK;
}

}  // namespace

extern "C" int cleave_verify(cleave_plan* plan, const void* A, int64_t lda, int transA,
                             const void* B, int64_t ldb, int transB, int dtype,
                             const float* partials, const float* r, const float* s, double tol,
                             double* lhs, double* rhs, double* scale, int32_t* accept,
                             void* hip_stream) {
  if (plan && plan->batch > 0) return CLEAVE_EINVAL;   // batched plans use the batched / grouped calls
  return verify_impl(plan, A, lda, transA, B, ldb, transB, dtype, partials, r, s, tol, lhs, rhs, scale,
                     accept, BatchLayout{}, hip_stream);
}

extern "C" int cleave_verify_reduce(cleave_plan* plan, const void* A, int64_t lda, int transA,
                                    const void* B, int64_t ldb, int transB, int dtype,
                                    const float* partials, const float* r, const float* s, double tol,
                                    double* lhs, double* rhs, double* scale, int32_t* accept,
                                    void* C, int64_t ldc, int out_dtype, void* hip_stream) {
  if (!plan || plan->batch > 0 || !C) return CLEAVE_EINVAL;
  if (out_dtype != CLEAVE_F32 && out_dtype != CLEAVE_BF16) return CLEAVE_EINVAL;
  if (ldc < plan->N || !aligned(C, out_dtype == CLEAVE_BF16 ? 2 : 4)) return CLEAVE_EINVAL;
  int rc = ensure_verify_tables_host(plan);
  if (rc != CLEAVE_OK) return rc;
  if (plan->verify->max_ksplit > static_cast<uint32_t>(cleave::kMaxFusedSplits)) {
    // more splits per tile than the fused pass carries: the two passes one after the other
    rc = verify_impl(plan, A, lda, transA, B, ldb, transB, dtype, partials, r, s, tol, lhs, rhs, scale,
                     accept, BatchLayout{}, hip_stream);
    if (rc != CLEAVE_OK) return rc;
    return reduce_impl(plan, partials, C, ldc, out_dtype, BatchLayout{}, hip_stream);
  }
  AggregateTarget agg;
  agg.C = C;
  agg.ldc = ldc;
  agg.out_dtype = out_dtype;
  return verify_impl(plan, A, lda, transA, B, ldb, transB, dtype, partials, r, s, tol, lhs, rhs, scale,
                     accept, BatchLayout{}, hip_stream, agg);
}

extern "C" int cleave_verify_batched(cleave_plan* plan, const void* A, int64_t lda, int transA,
                                     int64_t a_outer, int64_t a_inner, const void* B, int64_t ldb,
                                     int transB, int64_t b_outer, int64_t b_inner, int64_t n_inner,
                                     int dtype, const float* partials, const float* r, const float* s,
                                     double tol, double* lhs, double* rhs, double* scale,
                                     int32_t* accept, void* hip_stream) {
  if (!plan || plan->batch < 1) return CLEAVE_EINVAL;
  if (n_inner < 1 || n_inner > std::numeric_limits<uint32_t>::max() || plan->batch % n_inner != 0)
    return CLEAVE_EINVAL;
  if (a_outer < 0 || a_inner < 0 || b_outer < 0 || b_inner < 0) return CLEAVE_EINVAL;
  return verify_impl(plan, A, lda, transA, B, ldb, transB, dtype, partials, r, s, tol, lhs, rhs, scale,
                     accept, strided_layout(n_inner, a_outer, a_inner, b_outer, b_inner, 0, 0), hip_stream);
}

extern "C" int cleave_verify_grouped(cleave_plan* plan, int64_t n_members, const void* const* A_list,
                                     int64_t lda, int transA, const void* const* B_list, int64_t ldb,
                                     int transB, int dtype, const float* partials, const float* r,
                                     const float* s, double tol, double* lhs, double* rhs,
                                     double* scale, int32_t* accept, void* hip_stream) {
  if (!plan || plan->batch < 1 || plan->batch > cleave::kMaxGroup || n_members != plan->batch)
    return CLEAVE_EINVAL;
  if (dtype != CLEAVE_F32 && dtype != CLEAVE_BF16) return CLEAVE_EINVAL;
  const int eb = dtype == CLEAVE_BF16 ? 2 : 4;
  BatchLayout bl;
  bl.shape.n_group = static_cast<uint32_t>(plan->batch);
  const void* A = nullptr;
  const void* B = nullptr;
  int rc = group_offsets(A_list, plan->batch, eb, &bl.a, &A);
  if (rc != CLEAVE_OK) return rc;
  rc = group_offsets(B_list, plan->batch, eb, &bl.b, &B);
  if (rc != CLEAVE_OK) return rc;
  return verify_impl(plan, A, lda, transA, B, ldb, transB, dtype, partials, r, s, tol, lhs, rhs, scale,
                     accept, bl, hip_stream);
}
