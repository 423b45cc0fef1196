// Host-side task generation: row blocks of A x column blocks of B x chunks of
// the inner dimension (paper Sec. 3.2 "Seamless training", Sec. 4.1 "Search
// space of GEMM"; coverage and zero-task constraints of Sec. 4.1).
#include <algorithm>
#include <limits>
#include <new>

#include "plan_internal.h"

namespace cleave {

namespace {

struct Tile {
  int64_t m0, m_len, n0, n_len;
  int32_t ksplit;
};

constexpr int64_t kMaxDim = std::numeric_limits<int32_t>::max();

bool valid_split(int64_t K, int64_t S) {
  if (S < 1 || S > K) return false;
  const int64_t kc = (K + S - 1) / S;
  return (S - 1) * kc < K;
}

constexpr int kXcds = 8;
// A batch member with at least this many work items (one per CU of the chip) is
// spread over all XCDs instead of being kept on one.
constexpr size_t kSpreadItems = 256;

// The work items that run on an XCD at the same time (one per CU, 32 CUs) are
// taken from a patch of kPatchRows x kPatchCols sub-tiles at one chunk of the
// inner dimension: they share that many row panels of A and column panels of
// B in the XCD's L2.
#ifndef CLEAVE_PATCH_ROWS
#define CLEAVE_PATCH_ROWS 4
#endif
#ifndef CLEAVE_PATCH_COLS
#define CLEAVE_PATCH_COLS 8
#endif
constexpr uint32_t kPatchRows = CLEAVE_PATCH_ROWS;
constexpr uint32_t kPatchCols = CLEAVE_PATCH_COLS;

void order_work_items(cleave_plan* p) {
  // Region grid: minimise M/gm + N/gn over gm * gn = 8.
  int gm = 1, gn = kXcds;
  double best = 0.0;
  for (int g = 1; g <= kXcds; g *= 2) {
    const double cost = static_cast<double>(p->M) / g + static_cast<double>(p->N) / (kXcds / g);
    if (g == 1 || cost < best) {
      best = cost;
      gm = g;
      gn = kXcds / g;
    }
  }
  // three lists: the two classes of the mixed cut, then the all-small cut
  std::vector<WorkItem> all[kNumTileClasses], fine[kNumTileClasses];
  for (uint32_t i = 0; i < p->tasks.size(); ++i) {
    append_work_items(p->tasks[i], i, all);
    append_work_items(p->tasks[i], i, fine, true);
  }
  for (int list = 0; list < kNumTileClasses + 1; ++list) {
    const int cls = list < kNumTileClasses ? list : kTileSmall;
    const std::vector<WorkItem>& whole_list = list < kNumTileClasses ? all[cls] : fine[kTileSmall];
    std::vector<WorkItem>& ordered = list < kNumTileClasses ? p->items[cls] : p->items_fine;
    size_t& whole_steps = list < kNumTileClasses ? p->items_whole_steps[cls] : p->items_fine_whole_steps;
    ordered.reserve(whole_list.size());
    // Two parts, each ordered on its own: first the items the direct kernel
    // can take (chunk = whole K steps), then the others.
    for (int part = 0; part < 2; ++part) {
    std::vector<WorkItem> source;
    for (const WorkItem& w : whole_list)
      if ((w.k_len % kDirectKStep == 0) == (part == 0)) source.push_back(w);
    if (part == 0) whole_steps = source.size();
    if (source.empty()) continue;
    const uint32_t tr = static_cast<uint32_t>(tile_rows(cls));
    const uint32_t tc = static_cast<uint32_t>(tile_cols(cls));
    struct Key {
      uint32_t outer_member, split, pm, pn, inner_member, m, n;
      WorkItem item;
    };
    std::vector<Key> lists[kXcds];
    // Batch members share no output.  Small members (fewer items than the
    // chip has CUs) stay on one XCD each, member g on XCD g mod 8, one after
    // the other.  Large members (the GEMMs of one DAG level) are spread over
    // the XCDs like a single GEMM, and the members take turns patch by patch,
    // so that an operand panel they share is still in L2 for the next one.
    const bool member_per_xcd = p->batch > 0 && whole_list.size() / static_cast<size_t>(p->batch) < kSpreadItems;
    for (const WorkItem& w : source) {
      const cleave_task& t = p->tasks[w.task];
      const uint32_t m = w.m_base;
      const uint32_t n = w.n_base;
      const int rm = static_cast<int>(static_cast<uint64_t>(m) * gm / static_cast<uint64_t>(p->M));
      const int rn = static_cast<int>(static_cast<uint64_t>(n) * gn / static_cast<uint64_t>(p->N));
      // relative position of the chunk inside [0, K): tiles with different
      // split counts still line up by where in K they work
      const uint32_t split = static_cast<uint32_t>(static_cast<uint64_t>(t.k0) * 64 / static_cast<uint64_t>(p->K));
      const int region = member_per_xcd ? static_cast<int>(t.gemm_id % kXcds) : rm * gn + rn;
      lists[region].push_back(Key{member_per_xcd ? t.gemm_id : 0u, split, m / (kPatchRows * tr),
                                  n / (kPatchCols * tc), member_per_xcd ? 0u : t.gemm_id, m, n, w});
    }
    size_t longest = 0;
    for (auto& l : lists) {
      std::stable_sort(l.begin(), l.end(), [](const Key& a, const Key& b) {
        if (a.outer_member != b.outer_member) return a.outer_member < b.outer_member;
        if (a.split != b.split) return a.split < b.split;
        if (a.pm != b.pm) return a.pm < b.pm;
        if (a.pn != b.pn) return a.pn < b.pn;
        if (a.inner_member != b.inner_member) return a.inner_member < b.inner_member;
        if (a.m != b.m) return a.m < b.m;
        return a.n < b.n;
      });
      longest = std::max(longest, l.size());
    }
    // Interleave; when a region runs out, the slot is filled from the region
    // that has most left, so the list has no holes.
    size_t pos[kXcds] = {};
    for (size_t i = 0; i < longest; ++i) {
      for (int x = 0; x < kXcds; ++x) {
        int src = x;
        if (pos[src] >= lists[src].size()) {
          size_t most = 0;
          src = -1;
          for (int y = 0; y < kXcds; ++y) {
            const size_t left = lists[y].size() - pos[y];
            if (left > most) {
              most = left;
              src = y;
            }
          }
          if (src < 0) break;
        }
        ordered.push_back(lists[src][pos[src]++].item);
      }
    }
    for (int x = 0; x < kXcds; ++x)
      for (; pos[x] < lists[x].size(); ++pos[x]) ordered.push_back(lists[x][pos[x]].item);
    }
  }
}

// Emits the task records of `tiles` in canonical order and fills the derived
// tables.  Returns a status code.
// With n_batch > 0 the tile list is emitted n_batch times, once per batch
// member g, with gemm_id = g (tile ids restart, partial offsets run on).
int finish_plan(int64_t M, int64_t N, int64_t K, const std::vector<Tile>& tiles, uint32_t gemm_id,
                cleave_plan** out, int64_t n_batch = 0) {
  cleave_plan* p = new (std::nothrow) cleave_plan;
  if (!p) return CLEAVE_ENOMEM;
  try {
    const uint64_t copies = n_batch > 0 ? static_cast<uint64_t>(n_batch) : 1;
    p->M = M;
    p->N = N;
    p->K = K;
    p->batch = n_batch;
    p->num_tiles = static_cast<int64_t>(tiles.size() * copies);
    uint64_t off = 0;
    uint32_t tile_id = 0;
    // Task, tile and sub-tile indices are 32-bit in the task record and the
    // launch tables, offsets 64-bit: refuse a plan that does not fit rather
    // than wrap.
    constexpr uint64_t kMaxIndex = std::numeric_limits<uint32_t>::max();
    constexpr uint64_t kMaxElems = static_cast<uint64_t>(std::numeric_limits<int64_t>::max()) / 8;
    uint64_t n_tasks = 0;
    for (const Tile& tl : tiles) {
      n_tasks += static_cast<uint64_t>(tl.ksplit);
      const uint64_t subs = static_cast<uint64_t>((tl.m_len + kSmallTileRows - 1) / kSmallTileRows) *
                            static_cast<uint64_t>((tl.n_len + kSmallTileCols - 1) / kSmallTileCols);
      const uint64_t elems = static_cast<uint64_t>(tl.m_len) * static_cast<uint64_t>(tl.n_len);
      if (subs > kMaxIndex || n_tasks > kMaxIndex || elems > kMaxElems / static_cast<uint64_t>(tl.ksplit) ||
          (off += elems * static_cast<uint64_t>(tl.ksplit)) > kMaxElems) {
        delete p;
        return CLEAVE_EINVAL;
      }
    }
    if (n_tasks > kMaxIndex / copies || off > kMaxElems / copies) {
      delete p;
      return CLEAVE_EINVAL;
    }
    off = 0;
    for (uint64_t g = 0; g < copies; ++g) {
    if (n_batch > 0) gemm_id = static_cast<uint32_t>(g);
    tile_id = 0;
    for (const Tile& tl : tiles) {
      const int64_t S = tl.ksplit;
      const int64_t kc = (K + S - 1) / S;
      for (int64_t s = 0; s < S; ++s) {
        cleave_task t{};
        t.gemm_id = gemm_id;
        t.tile_id = tile_id;
        t.m0 = static_cast<uint32_t>(tl.m0);
        t.m_len = static_cast<uint32_t>(tl.m_len);
        t.n0 = static_cast<uint32_t>(tl.n0);
        t.n_len = static_cast<uint32_t>(tl.n_len);
        t.k0 = static_cast<uint32_t>(s * kc);
        t.k_len = static_cast<uint32_t>(std::min(kc, K - s * kc));
        t.ksplit_idx = static_cast<uint32_t>(s);
        t.ksplit_cnt = static_cast<uint32_t>(S);
        t.partial_off = off;
        off += static_cast<uint64_t>(tl.m_len) * static_cast<uint64_t>(tl.n_len);
        p->tasks.push_back(t);
      }
      ++tile_id;
    }
    }
    p->partial_elems = static_cast<int64_t>(off);
    p->seen_stamp.assign(p->tasks.size(), 0u);

    for (const cleave_task& t : p->tasks) {
      const uint32_t k_or = t.k0 | t.k_len;
      const uint32_t mn_or = t.m0 | t.m_len | t.n0 | t.n_len;
      p->all_k_mult8 &= (k_or % 8 == 0);
      p->all_k_mult4 &= (k_or % 4 == 0);
      p->all_mn_mult8 &= (mn_or % 8 == 0);
      p->all_mn_mult4 &= (mn_or % 4 == 0);
      p->all_n_mult4 &= ((t.n0 | t.n_len) % 4 == 0);
    }

    // Launch tables.  Execution order is free (only the task list's order is
    // part of the interface).  Workgroups are dispatched round-robin over the
    // 8 XCDs (workgroup b runs on XCD b % 8, each with its own L2), so work
    // item 8*i + x is the i-th item of XCD x.  Every XCD gets a compact
    // rectangle of the output (a gm x gn grid of regions with gm*gn = 8, chosen
    // to minimise the operand panels a region needs), and walks it chunk index
    // outermost: the items in flight on an XCD then share few row panels of A
    // and column panels of B, at the same chunk of the inner dimension.
    order_work_items(p);

    constexpr uint32_t kReduceElemsPerItem = 4096;
    for (uint32_t i = 0; i < p->tasks.size(); ++i) {
      const cleave_task& t = p->tasks[i];
      if (t.ksplit_idx != 0) continue;
      // a single split is a plain copy: fewer, longer items do better there
      const uint32_t elems = t.ksplit_cnt == 1 ? 4 * kReduceElemsPerItem : kReduceElemsPerItem;
      const uint32_t rows_per = std::max<uint32_t>(1, elems / t.n_len);
      for (uint32_t r = 0; r < t.m_len; r += rows_per) {
        p->reduce_items.push_back(ReduceItem{i, r, std::min(rows_per, t.m_len - r), 0});
      }
    }
  } catch (const std::bad_alloc&) {
    delete p;
    return CLEAVE_ENOMEM;
  }
  *out = p;
  return CLEAVE_OK;
}

}  // namespace

void balance_work_items(std::vector<WorkItem>& items, size_t n_direct, int grid,
                        std::vector<uint32_t>* ranges) {
  ranges->clear();
  if (grid < 2 || n_direct <= static_cast<size_t>(grid)) return;   // one item per workgroup at most
  const auto cost = [&](size_t i) { return work_item_cost(items[i]); };
  bool equal = true;
  for (size_t i = 1; i < n_direct && equal; ++i) equal = items[i].k_len == items[0].k_len;
  if (equal) return;

  std::vector<uint32_t> by_cost(n_direct);
  for (size_t i = 0; i < n_direct; ++i) by_cost[i] = static_cast<uint32_t>(i);
  std::stable_sort(by_cost.begin(), by_cost.end(),
                   [&](uint32_t a, uint32_t b) { return items[a].k_len > items[b].k_len; });
  std::vector<double> load(static_cast<size_t>(grid), 0.0);
  std::vector<std::vector<uint32_t>> owned(static_cast<size_t>(grid));
  for (uint32_t i : by_cost) {
    const int home = static_cast<int>(i % kXcds);
    int best_home = -1, best_any = 0;
    for (int b = 0; b < grid; ++b) {
      if (load[b] < load[best_any]) best_any = b;
      if (b % kXcds == home && (best_home < 0 || load[b] < load[best_home])) best_home = b;
    }
    const double c = cost(i);
    const int b = (best_home >= 0 && load[best_home] <= load[best_any] + c) ? best_home : best_any;
    load[b] += c;
    owned[b].push_back(i);
  }
  std::vector<WorkItem> out;
  out.reserve(n_direct);
  ranges->reserve(static_cast<size_t>(grid) + 1);
  for (int b = 0; b < grid; ++b) {
    ranges->push_back(static_cast<uint32_t>(out.size()));
    std::sort(owned[b].begin(), owned[b].end());
    for (uint32_t i : owned[b]) out.push_back(items[i]);
  }
  ranges->push_back(static_cast<uint32_t>(out.size()));
  std::copy(out.begin(), out.end(), items.begin());
}

void append_work_items(const cleave_task& t, uint32_t task_index, std::vector<WorkItem>* out,
                       bool fine) {
  const SubTiling s = sub_tiling(t, fine);
  for (uint32_t sub = 0; sub < s.count(); ++sub)
    out[s.cls].push_back(make_work_item(t, task_index, s, sub));
}

}  // namespace cleave

using cleave::Tile;

extern "C" int cleave_plan_uniform(int64_t M, int64_t N, int64_t K, int64_t tile_m, int64_t tile_n,
                                   int32_t ksplit, uint32_t gemm_id, cleave_plan** out) {
  if (!out) return CLEAVE_EINVAL;
  if (M < 1 || N < 1 || K < 1 || tile_m < 1 || tile_n < 1) return CLEAVE_EINVAL;
  if (M > cleave::kMaxDim || N > cleave::kMaxDim || K > cleave::kMaxDim) return CLEAVE_EINVAL;
  if (!cleave::valid_split(K, ksplit)) return CLEAVE_EINVAL;
  std::vector<Tile> tiles;
  try {
    for (int64_t m0 = 0; m0 < M; m0 += tile_m)
      for (int64_t n0 = 0; n0 < N; n0 += tile_n)
        tiles.push_back(Tile{m0, std::min(tile_m, M - m0), n0, std::min(tile_n, N - n0), ksplit});
  } catch (const std::bad_alloc&) {
    return CLEAVE_ENOMEM;
  }
  return cleave::finish_plan(M, N, K, tiles, gemm_id, out);
}

extern "C" int cleave_plan_batched(int64_t M, int64_t N, int64_t K, int64_t tile_m, int64_t tile_n,
                                   int32_t ksplit, int64_t n_batch, cleave_plan** out) {
  if (!out) return CLEAVE_EINVAL;
  if (M < 1 || N < 1 || K < 1 || tile_m < 1 || tile_n < 1 || n_batch < 1) return CLEAVE_EINVAL;
  if (M > cleave::kMaxDim || N > cleave::kMaxDim || K > cleave::kMaxDim ||
      n_batch > cleave::kMaxDim)
    return CLEAVE_EINVAL;
  if (!cleave::valid_split(K, ksplit)) return CLEAVE_EINVAL;
  std::vector<Tile> tiles;
  try {
    for (int64_t m0 = 0; m0 < M; m0 += tile_m)
      for (int64_t n0 = 0; n0 < N; n0 += tile_n)
        tiles.push_back(Tile{m0, std::min(tile_m, M - m0), n0, std::min(tile_n, N - n0), ksplit});
  } catch (const std::bad_alloc&) {
    return CLEAVE_ENOMEM;
  }
  return cleave::finish_plan(M, N, K, tiles, 0, out, n_batch);
}

extern "C" int cleave_plan_explicit(int64_t M, int64_t N, int64_t K, int32_t n_bands,
                                    const int64_t* band_h, const int32_t* n_cols,
                                    const int64_t* col_w, const int32_t* ksplit_per_tile,
                                    uint32_t gemm_id, cleave_plan** out) {
  if (!out || !band_h || !n_cols || !col_w || !ksplit_per_tile) return CLEAVE_EINVAL;
  if (M < 1 || N < 1 || K < 1 || n_bands < 1) return CLEAVE_EINVAL;
  if (M > cleave::kMaxDim || N > cleave::kMaxDim || K > cleave::kMaxDim) return CLEAVE_EINVAL;
  std::vector<Tile> tiles;
  try {
    int64_t m0 = 0;
    int64_t w_idx = 0;
    for (int32_t b = 0; b < n_bands; ++b) {
      const int64_t h = band_h[b];
      if (h < 1 || h > M - m0 || n_cols[b] < 1) return CLEAVE_EINVAL;
      int64_t n0 = 0;
      for (int32_t c = 0; c < n_cols[b]; ++c, ++w_idx) {
        const int64_t w = col_w[w_idx];
        if (w < 1 || w > N - n0) return CLEAVE_EINVAL;
        const int32_t S = ksplit_per_tile[tiles.size()];
        if (!cleave::valid_split(K, S)) return CLEAVE_EINVAL;
        tiles.push_back(Tile{m0, h, n0, w, S});
        n0 += w;
      }
      if (n0 != N) return CLEAVE_EINVAL;
      m0 += h;
    }
    if (m0 != M) return CLEAVE_EINVAL;
  } catch (const std::bad_alloc&) {
    return CLEAVE_ENOMEM;
  }
  return cleave::finish_plan(M, N, K, tiles, gemm_id, out);
}

extern "C" int64_t cleave_plan_num_tasks(const cleave_plan* plan) {
  return plan ? static_cast<int64_t>(plan->tasks.size()) : int64_t{CLEAVE_EINVAL};
}

extern "C" int64_t cleave_plan_num_tiles(const cleave_plan* plan) {
  return plan ? plan->num_tiles : int64_t{CLEAVE_EINVAL};
}

extern "C" const cleave_task* cleave_plan_tasks(const cleave_plan* plan) {
  return plan ? plan->tasks.data() : nullptr;
}

extern "C" int64_t cleave_plan_partial_elems(const cleave_plan* plan) {
  return plan ? plan->partial_elems : int64_t{CLEAVE_EINVAL};
}

extern "C" int cleave_plan_dims(const cleave_plan* plan, int64_t* dims) {
  if (!plan || !dims) return CLEAVE_EINVAL;
  dims[0] = plan->M;
  dims[1] = plan->N;
  dims[2] = plan->K;
  return CLEAVE_OK;
}

extern "C" const char* cleave_plan_last_kernel(const cleave_plan* plan) {
  return plan ? plan->last_kernel : "none";
}

extern "C" const char* cleave_strerror(int status) {
  switch (status) {
    case CLEAVE_OK: return "ok";
    case CLEAVE_EINVAL: return "invalid argument";
    case CLEAVE_ENOMEM: return "out of memory";
    case CLEAVE_EHIP: return "HIP runtime error";
    case CLEAVE_ELIMIT: return "request exceeds the fixed limit of this entry point";
    default: return "unknown status";
  }
}

extern "C" int cleave_plan_schedule_loads(const cleave_plan* plan, int list, int grid, int balanced,
                                          double* loads) {
  if (!plan || !loads || list < 0 || list > cleave::kNumTileClasses || grid < 1) return CLEAVE_EINVAL;
  const bool fine = list == cleave::kNumTileClasses;
  const std::vector<cleave::WorkItem>& host = fine ? plan->items_fine : plan->items[list];
  const size_t n_direct = fine ? plan->items_fine_whole_steps : plan->items_whole_steps[list];
  std::fill(loads, loads + grid, 0.0);
  try {
    std::vector<cleave::WorkItem> items(host.begin(), host.begin() + static_cast<std::ptrdiff_t>(n_direct));
    std::vector<uint32_t> ranges;
    if (balanced) cleave::balance_work_items(items, n_direct, grid, &ranges);
    if (!ranges.empty()) {
      for (int b = 0; b < grid; ++b)
        for (uint32_t i = ranges[b]; i < ranges[b + 1]; ++i) loads[b] += cleave::work_item_cost(items[i]);
    } else {
      for (size_t i = 0; i < n_direct; ++i) loads[i % static_cast<size_t>(grid)] += cleave::work_item_cost(items[i]);
    }
  } catch (const std::bad_alloc&) {
    return CLEAVE_ENOMEM;
  }
  return CLEAVE_OK;
}
