// Internal layout of a plan: host task list plus the launch tables derived
// from it, and their lazily created device copies.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>
#include <vector>

#include "cleave.h"

namespace cleave {

// Workgroup tile classes of the execute kernel.  Which class a task uses is a
// pure function of its record (see tile_class_of), so a re-issued task is cut
// into the same sub-tiles no matter which other tasks share the launch.
enum TileClass : int { kTileLarge = 0, kTileSmall = 1, kNumTileClasses = 2 };

#ifndef CLEAVE_LARGE_TILE_ROWS
#define CLEAVE_LARGE_TILE_ROWS 256
#endif
#ifndef CLEAVE_LARGE_TILE_COLS
#define CLEAVE_LARGE_TILE_COLS 256
#endif
constexpr int kLargeTileRows = CLEAVE_LARGE_TILE_ROWS;
constexpr int kLargeTileCols = CLEAVE_LARGE_TILE_COLS;
constexpr int kSmallTileRows = 128;
constexpr int kSmallTileCols = 128;

__host__ __device__ inline int tile_rows(int cls) { return cls == kTileLarge ? kLargeTileRows : kSmallTileRows; }
__host__ __device__ inline int tile_cols(int cls) { return cls == kTileLarge ? kLargeTileCols : kSmallTileCols; }

// Blocks with both edges above 128 are cut into large sub-tiles, everything
// else into 128 x 128 ones.
__host__ __device__ inline int tile_class_of(const cleave_task& t) {
  return (t.m_len > 128 && t.n_len > 128) ? kTileLarge : kTileSmall;
}

// One unit of work of the execute kernels: a sub-tile of one task's output
// block, computed over the task's whole chunk of the inner dimension.  The
// record carries everything a workgroup needs, so that one load -- issued well
// ahead -- replaces the dependent pair "which task, then that task's record".
// Elements of K the direct (global -> LDS) execute kernel consumes per step: it
// takes only items whose chunk length is a multiple of this.
constexpr uint32_t kDirectKStep = 64;

struct alignas(16) WorkItem {
  uint32_t m_base, n_base;    // first row / column of the sub-tile in the logical output
  uint32_t k0, k_len;         // the task's chunk
  uint32_t m_valid, n_valid;  // extent of the sub-tile (at most the class's tile)
  uint32_t out_ld;            // row stride of the task's partial block (= its n_len)
  uint32_t gemm_id;           // batch member (batched plans)
  uint64_t out_off;           // element offset of the sub-tile's origin in the partial buffer
  uint32_t task;              // index into the task table
  uint32_t sub;               // sub-tile index within the task's block, row-major
};
static_assert(sizeof(WorkItem) == 48, "WorkItem is 48 bytes");

// How a task's block is cut into sub-tiles: the class (or, with `fine`, the
// small class for every block) fixes the sub-tile, the block's extent the grid
// of sub-tiles.  Host and device share this one definition.
struct SubTiling {
  int cls;
  uint32_t tr, tc;    // sub-tile rows / columns
  uint32_t sm, sn;    // grid of sub-tiles
  __host__ __device__ uint32_t count() const { return sm * sn; }
};
__host__ __device__ inline SubTiling sub_tiling(const cleave_task& t, bool fine) {
  SubTiling s;
  s.cls = fine ? static_cast<int>(kTileSmall) : tile_class_of(t);
  s.tr = static_cast<uint32_t>(tile_rows(s.cls));
  s.tc = static_cast<uint32_t>(tile_cols(s.cls));
  s.sm = (t.m_len + s.tr - 1) / s.tr;
  s.sn = (t.n_len + s.tc - 1) / s.tc;
  return s;
}
// Work item of sub-tile `sub` (row-major in the grid) of task record t.
__host__ __device__ inline WorkItem make_work_item(const cleave_task& t, uint32_t task_index,
                                                   const SubTiling& s, uint32_t sub) {
  const uint32_t i = sub / s.sn, j = sub - i * s.sn;
  WorkItem w{};
  w.m_base = t.m0 + i * s.tr;
  w.n_base = t.n0 + j * s.tc;
  w.k0 = t.k0;
  w.k_len = t.k_len;
  w.m_valid = s.tr < t.m_len - i * s.tr ? s.tr : t.m_len - i * s.tr;
  w.n_valid = s.tc < t.n_len - j * s.tc ? s.tc : t.n_len - j * s.tc;
  w.out_ld = t.n_len;
  w.gemm_id = t.gemm_id;
  w.out_off = t.partial_off + static_cast<uint64_t>(i) * s.tr * t.n_len + static_cast<uint64_t>(j) * s.tc;
  w.task = task_index;
  w.sub = sub;
  return w;
}

// One unit of work of the reduce kernel: a run of rows of one output tile.
struct ReduceItem {
  uint32_t task;    // index of the tile's chunk-0 task
  uint32_t row0;    // first row within the tile
  uint32_t rows;    // number of rows
  uint32_t pad;
};
static_assert(sizeof(ReduceItem) == 16, "ReduceItem is 16 bytes");

// Tables of the returned-block check.  A row segment is a distinct (m0, m_len)
// of the task list, a column segment a distinct (n0, n_len): the projections
// of A onto r and of B onto s are computed once per segment and shared by all
// tasks that use it.
struct Segment {
  uint32_t start, len;
};
// One unit of work of the bilinear-form kernel: a run of rows of one task's
// partial block.
struct VerifyItem {
  uint32_t task, row0, rows;
  uint32_t slot;   // fused pass only: where the item's sum for the tile's first split goes
};
static_assert(sizeof(VerifyItem) == 16, "VerifyItem is 16 bytes");

struct VerifyTables {
  std::vector<Segment> row_segs, col_segs;
  std::vector<uint32_t> task_row_seg, task_col_seg;   // per task
  std::vector<VerifyItem> items;                      // a task's items are adjacent
  std::vector<uint32_t> task_first_item;              // n_tasks + 1 entries
  // Fused check + aggregation: its own, shorter items (runs of rows of a tile,
  // taken for all splits at once; listed for the first split's task only) and
  // the slots their sums go to (a task's slots are adjacent, as above).
  std::vector<VerifyItem> agg_items;
  std::vector<uint32_t> agg_first_item;               // n_tasks + 1 entries
  uint32_t max_ksplit = 1;
  bool segs_mult8 = true;   // every segment start and length a multiple of 8
  bool segs_mult4 = true;
  // device copies and scratch (allocated once, on the device the plan lives on)
  Segment* d_row_segs = nullptr;
  Segment* d_col_segs = nullptr;
  uint32_t* d_task_row_seg = nullptr;
  uint32_t* d_task_col_seg = nullptr;
  VerifyItem* d_items = nullptr;
  uint32_t* d_task_first_item = nullptr;
  VerifyItem* d_agg_items = nullptr;
  uint32_t* d_agg_first_item = nullptr;
  double* d_agg_item_sums = nullptr;
  double* d_proj = nullptr;       // U, |U| (row segs x K each), V, |V| (col segs x K each)
  double* d_item_sums = nullptr;  // one per item
};

// Device memory the subset launches of a plan put their work-item lists in.
// Sized when the plan's tables are uploaded; nothing is allocated later.
//   eager calls:    slices of a ring of 2 * max_items items; a slice is reused
//                   only after the launch that read it has finished (one event
//                   per launch; the host waits only if the ring has wrapped
//                   onto a launch that is still running);
//   captured calls: (the stream is being captured into a HIP graph) slices of a
//                   second buffer of max_items items that are never reused,
//                   since a graph may be replayed as long as the plan lives.
// max_items = the plan's own work-item count under its finest cut, which no
// subset exceeds.
struct SubsetRing {
  WorkItem* d_ring = nullptr;
  WorkItem* d_captured = nullptr;
  int64_t max_items = 0;
  int64_t pos = 0;             // next free item of the ring
  int64_t captured_used = 0;   // items of d_captured handed out
  struct InFlight {
    int64_t begin, end;
    hipEvent_t done;
  };
  std::vector<InFlight> in_flight;       // oldest first
  std::vector<hipEvent_t> idle_events;
  std::mutex mu;                         // subset calls of one plan may come from several threads
};

// Appends the work items of `task_index` (record t) to out[class].  With
// `fine` every block is cut into small-class sub-tiles.  Either cut gives the
// same bits: both kernels shapes accumulate an output element in the same
// order (ascending K steps and sub-steps), so the choice is free per launch.
// Workgroup schedule for a list of work items of unequal length (heterogeneous
// tilings: Sec. 4.1 gives every device its own shard size, Sec. 3.2 its own
// split of the inner dimension).  The persistent kernel's default -- workgroup
// b takes items b, b + grid, ... -- leaves the workgroups with very different
// totals when chunk lengths differ by a factor of eight.  This reorders the
// first n_direct items so that workgroup b owns the contiguous run
// [ranges[b], ranges[b + 1]) and the runs have nearly equal cost: longest items
// first, each to the least-loaded workgroup of the XCD the item's position
// belongs to (position mod 8, as the list was laid out) unless a workgroup of
// another XCD is behind by more than the item's own cost; inside a run the
// original order is kept.  Returns with `ranges` empty, and the list
// untouched, when all items cost the same or no workgroup gets a second item.
void balance_work_items(std::vector<WorkItem>& items, size_t n_direct, int grid,
                        std::vector<uint32_t>* ranges);
// Cost of a work item in the schedule's unit (one K step of the fast kernel):
// its K steps plus a constant for the store phase (measured: 12 K clocks
// against 2.6 K per step).
inline double work_item_cost(const WorkItem& w) {
  return w.k_len / kDirectKStep + 4.5;
}

void append_work_items(const cleave_task& t, uint32_t task_index, std::vector<WorkItem>* out,
                       bool fine = false);

}  // namespace cleave

struct cleave_plan {
  int64_t M = 0, N = 0, K = 0;
  int64_t partial_elems = 0;
  int64_t num_tiles = 0;
  int64_t batch = 0;         // > 0: a batch of that many M x N x K GEMMs, task.gemm_id = member
  bool all_k_mult8 = true;   // every k0 and k_len is a multiple of 8
  bool all_k_mult4 = true;
  bool all_mn_mult8 = true;  // every m0, m_len, n0, n_len is a multiple of 8
  bool all_mn_mult4 = true;
  bool all_n_mult4 = true;   // every n0, n_len multiple of 4 (vector path of reduce)
  std::vector<cleave_task> tasks;
  // All tasks, launch order.  Each list starts with the items whose chunk is a
  // whole number of the direct kernel's K steps (items_whole_steps of them);
  // the rest can only run in the staged kernel.
  std::vector<cleave::WorkItem> items[cleave::kNumTileClasses];
  size_t items_whole_steps[cleave::kNumTileClasses] = {0, 0};
  // All tasks cut into small-class sub-tiles only: used when the large class
  // would leave most of the CUs without a work item.
  std::vector<cleave::WorkItem> items_fine;
  size_t items_fine_whole_steps = 0;
  std::vector<cleave::ReduceItem> reduce_items;

  // Device copies (current device at first use).
  int device = -1;
  cleave_task* d_tasks = nullptr;
  cleave::WorkItem* d_items[cleave::kNumTileClasses] = {nullptr, nullptr};
  cleave::WorkItem* d_items_fine = nullptr;
  // Balanced schedules of the three lists' direct parts (large, small, fine) for
  // the grid sizes of the device the tables were uploaded to; null = equal items.
  uint32_t* d_wg_ranges[cleave::kNumTileClasses + 1] = {nullptr, nullptr, nullptr};
  int wg_ranges_grid[cleave::kNumTileClasses + 1] = {0, 0, 0};
  cleave::ReduceItem* d_reduce_items = nullptr;
  // Work-item slices of subset launches (device memory sized once, at upload).
  cleave::SubsetRing subset;
  // Repeat check of a subset's task ids without clearing or allocating: task i
  // was listed in the current call iff seen_stamp[i] == seen_generation (one
  // entry per task, made with the plan; guarded by subset.mu).
  std::vector<uint32_t> seen_stamp;
  uint32_t seen_generation = 0;

  // Tables and scratch of the returned-block check; created by its first call.
  cleave::VerifyTables* verify = nullptr;

  const char* last_kernel = "none";
};
