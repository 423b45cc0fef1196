// Host-side cost model and heterogeneous shard assignment (paper Sec. 4.1
// "Optimization Problem and its Cost Model"; Sec. 4.2 for the cache-aware
// downlink term).  The step right before the hot path: its output is exactly
// the input of cleave_plan_explicit (row bands, column widths per band) plus
// the device that owns each tile.
//
// The paper hands the assignment to a MILP solver.  Here it is a deterministic
// construction inside a bisection on the target time T:
//   * a device's edge e_k(T) is the largest multiple of the granule whose
//     square shard costs at most T and fits the device's memory;
//   * devices are taken by descending edge; a row band takes the height of
//     the next device (clipped to the rows left) and is cut into columns left
//     to right, every next device getting the widest shard that costs at most
//     T at that height; devices that cannot take a granule stay idle;
//   * T is feasible when the rows are covered before the devices run out.
// Every comparison is made in IEEE double precision on expressions evaluated
// in a fixed order (no contraction), so the layout is a pure function of the
// inputs.
#include <algorithm>
#include <cstdint>
#include <new>
#include <numeric>
#include <utility>
#include <vector>

#include "cleave.h"

namespace {

struct Layout {
  std::vector<int64_t> band_h;
  std::vector<int32_t> n_cols;
  std::vector<int64_t> col_w;      // band-major
  std::vector<int32_t> owner;      // band-major
};

double cost_of(const cleave_device& d, int64_t alpha, int64_t beta, int64_t alpha_fetch,
               int64_t beta_fetch, int64_t n, int64_t b) {
  if (alpha == 0 && beta == 0) return 0.0;
  const double c_dl = static_cast<double>(alpha_fetch * n * b + n * beta_fetch * b) / d.down_bw + d.down_lat;
  const double c_ul = static_cast<double>(alpha * beta * b) / d.up_bw + d.up_lat;
  const double c_comp = static_cast<double>(2 * alpha * beta * n) / d.flops;
  return std::max(std::max(c_dl, c_ul), c_comp);
}

bool fits(const cleave_device& d, int64_t alpha, int64_t beta, int64_t n, int64_t b) {
  return static_cast<double>(alpha * n * b + n * beta * b + alpha * beta * b) <= d.mem_bytes;
}

// Largest u in [0, limit] for which ok(u) holds; ok is true up to some point and false after.
template <typename F>
int64_t largest(int64_t limit, F ok) {
  int64_t lo = 0, hi = limit;
  while (lo < hi) {
    const int64_t mid = (lo + hi + 1) / 2;
    if (ok(mid)) lo = mid;
    else hi = mid - 1;
  }
  return lo;
}

// What the survivors of a device failure already hold (churn recovery,
// Sec. 4.2: the binary cache matrices R_s and C_s): per device the set of rows
// of A and the set of columns of B it has cached, each as a list of disjoint
// half-open intervals in absolute output coordinates (a row of R_s / C_s with
// its runs of ones written as intervals), the bytes of its memory already in
// use (no cache replacement), and where the rectangle to cover starts.
// `on` false: cold start.
struct IntervalSet {
  const int64_t* iv = nullptr;   // n pairs [lo, hi)
  int32_t n = 0;
};
struct Caches {
  bool on = false;
  std::vector<IntervalSet> rows, cols;   // one per device
  const double* mem_used = nullptr;      // one per device
  int64_t row0 = 0, col0 = 0;
};

int64_t overlap(int64_t lo, int64_t hi, int64_t c_lo, int64_t c_hi) {
  return std::max<int64_t>(0, std::min(hi, c_hi) - std::max(lo, c_lo));
}

// Elements of [lo, hi) that the set holds.
int64_t covered(const IntervalSet& s, int64_t lo, int64_t hi) {
  int64_t total = 0;
  for (int32_t i = 0; i < s.n; ++i) total += overlap(lo, hi, s.iv[2 * i], s.iv[2 * i + 1]);
  return total;
}

bool build_layout(int64_t m, int64_t q, int64_t n, int64_t b, const cleave_device* devs,
                  int32_t n_devs, int64_t g, double T, const Caches& cc, Layout* out) {
  const int64_t top = (std::max(m, q) + g - 1) / g;
  // rows / columns of a shard at (r_lo, c_lo) of the rectangle that device k must still fetch
  auto fetch = [&](int32_t k, int64_t r_lo, int64_t h, int64_t c_lo, int64_t w, int64_t* af, int64_t* bf) {
    if (!cc.on) {
      *af = h;
      *bf = w;
      return;
    }
    const int64_t a_lo = cc.row0 + r_lo, b_lo = cc.col0 + c_lo;
    *af = h - covered(cc.rows[k], a_lo, a_lo + h);
    *bf = w - covered(cc.cols[k], b_lo, b_lo + w);
  };
  auto affordable = [&](int32_t k, int64_t h, int64_t w, int64_t af, int64_t bf) {
    const cleave_device& d = devs[k];
    if (cost_of(d, h, w, af, bf, n, b) > T) return false;
    if (!cc.on) return fits(d, h, w, n, b);
    return static_cast<double>(af * n * b + n * bf * b + h * w * b) + cc.mem_used[k] <= d.mem_bytes;
  };
  std::vector<int64_t> edge(n_devs);
  for (int32_t k = 0; k < n_devs; ++k) {
    // the shard's position is not known yet: every cached row and column of the
    // rectangle counts as if the shard were placed on it
    int64_t hr = 0, hc = 0;
    if (cc.on) {
      hr = covered(cc.rows[k], cc.row0, cc.row0 + m);
      hc = covered(cc.cols[k], cc.col0, cc.col0 + q);
    }
    edge[k] = g * largest(top, [&](int64_t u) {
                const int64_t e = u * g;
                return affordable(k, e, e, std::max<int64_t>(0, e - hr), std::max<int64_t>(0, e - hc));
              });
  }
  std::vector<int32_t> order;
  for (int32_t k = 0; k < n_devs; ++k)
    if (edge[k] > 0) order.push_back(k);
  std::stable_sort(order.begin(), order.end(),
                   [&](int32_t x, int32_t y) { return edge[x] > edge[y]; });   // ties keep index order
  out->band_h.clear();
  out->n_cols.clear();
  out->col_w.clear();
  out->owner.clear();
  size_t pos = 0;
  int64_t rows_left = m;
  while (rows_left > 0) {
    if (pos >= order.size()) return false;
    const int64_t h = std::min(edge[order[pos]], rows_left);
    int32_t cols = 0;
    int64_t cols_left = q;
    while (cols_left > 0) {
      if (pos >= order.size()) return false;
      const int32_t k = order[pos++];
      const int64_t r_lo = m - rows_left, c_lo = q - cols_left;
      const int64_t units = largest((cols_left + g - 1) / g, [&](int64_t u) {
        const int64_t w = std::min(u * g, cols_left);
        int64_t af, bf;
        fetch(k, r_lo, h, c_lo, w, &af, &bf);
        return affordable(k, h, w, af, bf);
      });
      const int64_t w = std::min(units * g, cols_left);
      if (w == 0) continue;   // this device stays idle
      out->col_w.push_back(w);
      out->owner.push_back(k);
      ++cols;
      cols_left -= w;
    }
    out->band_h.push_back(h);
    out->n_cols.push_back(cols);
    rows_left -= h;
  }
  return true;
}

bool valid_device(const cleave_device& d) {
  return d.down_bw > 0.0 && d.up_bw > 0.0 && d.flops > 0.0 && d.down_lat >= 0.0 && d.up_lat >= 0.0 &&
         d.mem_bytes >= 0.0;
}

// Sizes for which every integer expression of the cost model stays below 2^53.
bool sizes_ok(int64_t m, int64_t q, int64_t n, int64_t b) {
  constexpr int64_t kMax = int64_t{1} << 24;
  return m >= 1 && q >= 1 && n >= 1 && b >= 1 && m <= kMax && q <= kMax && n <= kMax && b <= 16;
}

}  // namespace

extern "C" double cleave_shard_cost(const cleave_device* dev, int64_t alpha, int64_t beta,
                                    int64_t alpha_fetch, int64_t beta_fetch, int64_t n,
                                    int32_t elem_bytes) {
  if (!dev || !valid_device(*dev) || alpha < 0 || beta < 0 || (alpha == 0) != (beta == 0) ||
      alpha_fetch < 0 || beta_fetch < 0 || alpha_fetch > alpha || beta_fetch > beta ||
      !sizes_ok(std::max<int64_t>(alpha, 1), std::max<int64_t>(beta, 1), n, elem_bytes))
    return -1.0;
  return cost_of(*dev, alpha, beta, alpha_fetch, beta_fetch, n, elem_bytes);
}

extern "C" int cleave_shard_fits(const cleave_device* dev, int64_t alpha, int64_t beta, int64_t n,
                                 int32_t elem_bytes) {
  if (!dev || !valid_device(*dev) || alpha < 0 || beta < 0 ||
      !sizes_ok(std::max<int64_t>(alpha, 1), std::max<int64_t>(beta, 1), n, elem_bytes))
    return CLEAVE_EINVAL;
  return fits(*dev, alpha, beta, n, elem_bytes) ? 1 : 0;
}

namespace {

int assign_impl(int64_t m, int64_t q, int64_t n, int32_t elem_bytes, const cleave_device* devs,
                int32_t n_devs, int64_t granule, const Caches& cc, int32_t* n_bands, int64_t* band_h,
                int32_t* n_cols, int64_t* col_w, int32_t* tile_device, double* cost) {
  if (!devs || !n_bands || !band_h || !n_cols || !col_w || !tile_device || !cost) return CLEAVE_EINVAL;
  if (n_devs < 1 || granule < 1 || !sizes_ok(m, q, n, elem_bytes)) return CLEAVE_EINVAL;
  for (int32_t k = 0; k < n_devs; ++k)
    if (!valid_device(devs[k])) return CLEAVE_EINVAL;
  try {
    Layout found, trial;
    double t_hi = 1e-9;
    bool ok = false;
    for (int i = 0; i < 80 && !ok; ++i) {
      ok = build_layout(m, q, n, elem_bytes, devs, n_devs, granule, t_hi, cc, &found);
      if (!ok) t_hi *= 2.0;
    }
    if (!ok) return CLEAVE_EINVAL;   // the memory capacities admit no cover
    double lo = 0.0, hi = t_hi;
    for (int i = 0; i < 64; ++i) {
      const double mid = (lo + hi) / 2.0;
      if (build_layout(m, q, n, elem_bytes, devs, n_devs, granule, mid, cc, &trial)) {
        hi = mid;
        std::swap(found, trial);
      } else {
        lo = mid;
      }
    }
    double worst = 0.0;
    size_t t = 0;
    int64_t r_lo = 0;
    for (size_t band = 0; band < found.band_h.size(); ++band) {
      int64_t c_lo = 0;
      const int64_t h = found.band_h[band];
      for (int32_t c = 0; c < found.n_cols[band]; ++c, ++t) {
        const int64_t w = found.col_w[t];
        int64_t af = h, bf = w;
        if (cc.on) {
          af = h - covered(cc.rows[found.owner[t]], cc.row0 + r_lo, cc.row0 + r_lo + h);
          bf = w - covered(cc.cols[found.owner[t]], cc.col0 + c_lo, cc.col0 + c_lo + w);
        }
        worst = std::max(worst, cost_of(devs[found.owner[t]], h, w, af, bf, n, elem_bytes));
        c_lo += w;
      }
      r_lo += h;
    }
    *n_bands = static_cast<int32_t>(found.band_h.size());
    std::copy(found.band_h.begin(), found.band_h.end(), band_h);
    std::copy(found.n_cols.begin(), found.n_cols.end(), n_cols);
    std::copy(found.col_w.begin(), found.col_w.end(), col_w);
    std::copy(found.owner.begin(), found.owner.end(), tile_device);
    *cost = worst;
  } catch (const std::bad_alloc&) {
    return CLEAVE_ENOMEM;
  }
  return CLEAVE_OK;
}

}  // namespace

extern "C" int cleave_assign(int64_t m, int64_t q, int64_t n, int32_t elem_bytes,
                             const cleave_device* devs, int32_t n_devs, int64_t granule,
                             int32_t* n_bands, int64_t* band_h, int32_t* n_cols, int64_t* col_w,
                             int32_t* tile_device, double* cost) {
  return assign_impl(m, q, n, elem_bytes, devs, n_devs, granule, Caches{}, n_bands, band_h, n_cols,
                     col_w, tile_device, cost);
}

namespace {

// Sorted, disjoint, non-negative, non-inverted intervals.
bool valid_set(const IntervalSet& s) {
  int64_t prev_hi = 0;
  for (int32_t i = 0; i < s.n; ++i) {
    const int64_t lo = s.iv[2 * i], hi = s.iv[2 * i + 1];
    if (lo < prev_hi || hi < lo) return false;
    prev_hi = hi;
  }
  return true;
}

}  // namespace

extern "C" int cleave_reassign(int64_t m, int64_t q, int64_t n, int32_t elem_bytes,
                               const cleave_device* devs, int32_t n_devs, int64_t granule,
                               int64_t row0, int64_t col0, const int64_t* cached,
                               const double* mem_used, int32_t* n_bands, int64_t* band_h,
                               int32_t* n_cols, int64_t* col_w, int32_t* tile_device, double* cost) {
  if (!cached || !mem_used || row0 < 0 || col0 < 0 || n_devs < 1) return CLEAVE_EINVAL;
  Caches cc;
  try {
    cc.rows.resize(static_cast<size_t>(n_devs));
    cc.cols.resize(static_cast<size_t>(n_devs));
  } catch (const std::bad_alloc&) {
    return CLEAVE_ENOMEM;
  }
  for (int32_t k = 0; k < n_devs; ++k) {
    const int64_t* c = cached + 4 * static_cast<int64_t>(k);
    if (c[0] < 0 || c[1] < c[0] || c[2] < 0 || c[3] < c[2] || !(mem_used[k] >= 0.0)) return CLEAVE_EINVAL;
    cc.rows[k] = IntervalSet{c, 1};
    cc.cols[k] = IntervalSet{c + 2, 1};
  }
  cc.on = true;
  cc.mem_used = mem_used;
  cc.row0 = row0;
  cc.col0 = col0;
  return assign_impl(m, q, n, elem_bytes, devs, n_devs, granule, cc, n_bands, band_h, n_cols, col_w,
                     tile_device, cost);
}

extern "C" int cleave_reassign_sets(int64_t m, int64_t q, int64_t n, int32_t elem_bytes,
                                    const cleave_device* devs, int32_t n_devs, int64_t granule,
                                    int64_t row0, int64_t col0, const int32_t* n_row_iv,
                                    const int64_t* row_iv, const int32_t* n_col_iv,
                                    const int64_t* col_iv, const double* mem_used, int32_t* n_bands,
                                    int64_t* band_h, int32_t* n_cols, int64_t* col_w,
                                    int32_t* tile_device, double* cost) {
  if (!n_row_iv || !n_col_iv || !mem_used || row0 < 0 || col0 < 0 || n_devs < 1) return CLEAVE_EINVAL;
  Caches cc;
  try {
    cc.rows.resize(static_cast<size_t>(n_devs));
    cc.cols.resize(static_cast<size_t>(n_devs));
  } catch (const std::bad_alloc&) {
    return CLEAVE_ENOMEM;
  }
  int64_t r_at = 0, c_at = 0;
  for (int32_t k = 0; k < n_devs; ++k) {
    if (n_row_iv[k] < 0 || n_col_iv[k] < 0 || !(mem_used[k] >= 0.0)) return CLEAVE_EINVAL;
    if ((n_row_iv[k] > 0 && !row_iv) || (n_col_iv[k] > 0 && !col_iv)) return CLEAVE_EINVAL;
    cc.rows[k] = IntervalSet{row_iv ? row_iv + 2 * r_at : nullptr, n_row_iv[k]};
    cc.cols[k] = IntervalSet{col_iv ? col_iv + 2 * c_at : nullptr, n_col_iv[k]};
    if (!valid_set(cc.rows[k]) || !valid_set(cc.cols[k])) return CLEAVE_EINVAL;
    r_at += n_row_iv[k];
    c_at += n_col_iv[k];
  }
  cc.on = true;
  cc.mem_used = mem_used;
  cc.row0 = row0;
  cc.col0 = col0;
  return assign_impl(m, q, n, elem_bytes, devs, n_devs, granule, cc, n_bands, band_h, n_cols, col_w,
                     tile_device, cost);
}
