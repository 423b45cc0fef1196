"""Reference for the cost model of Sec. 4.1 and a heterogeneous shard
assignment built on it -- TEST INFRASTRUCTURE ONLY (same rule as the rest of
this package).

Cost model (Sec. 4.1, "Communication cost", "Computation cost", "Cost model
constraints"), for device k and a shard of alpha rows of A (m x n) and beta
columns of B (n x q), element size b bytes:
    C_dl   = (alpha n b + n beta b) / W_dl + L_dl
    C_ul   = alpha beta b / W_ul + L_ul
    C_comp = 2 alpha beta n / F
    C      = max(C_dl, C_ul, C_comp)            downlink, uplink, compute overlap
    memory:  alpha n b + n beta b + alpha beta b <= Mem
    a device is either idle (alpha = beta = 0) or has alpha, beta >= 1
    the shards of a GEMM cover its m x q output exactly once
    GEMM cost = max over devices; churn recovery (Sec. 4.2) replaces alpha, beta
    in C_dl by the rows / columns the device still has to fetch.

The paper solves the assignment with a commercial MILP solver; this reference
takes a deterministic heuristic instead (stated here in full, because the
library's planner is tested for producing the same layout):

  feasible(T): each device's edge e_k = largest multiple of the granule g (at
  most max(m, q) rounded up) with C(e_k, e_k) <= T and the memory constraint
  (in a churn re-solve, with the rows and columns of the rectangle that the
  device already holds counted as not to be fetched);
  devices are ordered by e_k descending (index ascending on ties), devices
  with e_k = 0 stay idle.  Row bands are cut top to bottom: a band takes the
  next unused device, its height is h = min(e_k, rows left); inside the band
  columns are cut left to right, each next unused device getting the largest
  width w (multiple of g, at most the columns left, which may be a ragged
  rest) with C(h, w) <= T and the memory constraint; a device whose w is 0 is
  skipped (idle).  T is feasible when all rows are covered before the devices
  run out.
  T* is found by bisection on [0, T_hi], 64 halvings, T_hi = the smallest T of
  the form 2^j * 1e-9 s that is feasible; the layout of the last feasible T is
  returned with its true cost max_k C(alpha_k, beta_k).
All decisions are taken in IEEE double precision with the expression order
written below, so that an independent implementation reproduces the layout
bit for bit.
"""
import math


class Device:
    __slots__ = ("down_bw", "up_bw", "down_lat", "up_lat", "flops", "mem_bytes")

    def __init__(self, down_bw, up_bw, down_lat, up_lat, flops, mem_bytes):
        self.down_bw = float(down_bw)     # bytes / s
        self.up_bw = float(up_bw)
        self.down_lat = float(down_lat)   # s
        self.up_lat = float(up_lat)
        self.flops = float(flops)         # flop / s
        self.mem_bytes = float(mem_bytes)


def shard_cost(dev, alpha, beta, n, b, alpha_fetch=None, beta_fetch=None):
    """C(alpha, beta) for one device; idle shard costs 0.  alpha_fetch /
    beta_fetch: rows / columns still to download (churn recovery), default all."""
    if alpha == 0 and beta == 0:
        return 0.0
    if alpha < 1 or beta < 1:
        raise ValueError("a shard has rows and columns, or neither")
    af = alpha if alpha_fetch is None else alpha_fetch
    bf = beta if beta_fetch is None else beta_fetch
    c_dl = float(af * n * b + n * bf * b) / dev.down_bw + dev.down_lat
    c_ul = float(alpha * beta * b) / dev.up_bw + dev.up_lat
    c_comp = float(2 * alpha * beta * n) / dev.flops
    return max(max(c_dl, c_ul), c_comp)


def shard_fits(dev, alpha, beta, n, b):
    return float(alpha * n * b + n * beta * b + alpha * beta * b) <= dev.mem_bytes


def _largest(limit_units, g, ok):
    """Largest u in [0, limit_units] with ok(u * g) (ok is monotone: true up to a point)."""
    lo, hi = 0, limit_units
    while lo < hi:
        mid = (lo + hi + 1) // 2
        if ok(mid * g):
            lo = mid
        else:
            hi = mid - 1
    return lo


def _overlap(lo, hi, c_lo, c_hi):
    return max(0, min(hi, c_hi) - max(lo, c_lo))


def _covered(intervals, lo, hi):
    """Elements of [lo, hi) inside a list of disjoint half-open intervals."""
    return sum(_overlap(lo, hi, a, b) for a, b in intervals)


def _as_sets(entry):
    """A device's cache: (row_lo, row_hi, col_lo, col_hi) -- one interval each --
    or (row_intervals, col_intervals) with lists of (lo, hi) pairs, the runs of
    ones of the device's rows in the cache matrices R_s and C_s (Sec. 4.2)."""
    if len(entry) == 4:
        return [(entry[0], entry[1])], [(entry[2], entry[3])]
    return list(entry[0]), list(entry[1])


def _layout(m, q, n, b, devs, g, T, origin=(0, 0), cached=None, mem_used=None):
    """The construction for target time T; returns None if the devices run out.

    Churn recovery (Sec. 4.2): `cached[k]` = (row_lo, row_hi, col_lo, col_hi), the
    rows of A and columns of B device k already holds (absolute indices; the
    rectangle to cover starts at `origin`), which it need not download again;
    `mem_used[k]` = bytes of its memory already taken (no cache replacement)."""
    top = -(-max(m, q) // g)

    def cost_at(k, r_lo, h, c_lo, w):
        d = devs[k]
        if cached is None:
            return shard_cost(d, h, w, n, b)
        rows, cols = _as_sets(cached[k])
        a_lo, c0 = origin[0] + r_lo, origin[1] + c_lo
        return shard_cost(d, h, w, n, b, h - _covered(rows, a_lo, a_lo + h), w - _covered(cols, c0, c0 + w))

    def fits_at(k, r_lo, h, c_lo, w):
        d = devs[k]
        if cached is None:
            return shard_fits(d, h, w, n, b)
        rows, cols = _as_sets(cached[k])
        a_lo, c0 = origin[0] + r_lo, origin[1] + c_lo
        af = h - _covered(rows, a_lo, a_lo + h)
        bf = w - _covered(cols, c0, c0 + w)
        return float(af * n * b + n * bf * b + h * w * b) + mem_used[k] <= d.mem_bytes

    edges = []
    for k, d in enumerate(devs):
        # the shard's position is not known yet: the edge counts every cached row
        # and column of the rectangle as if the shard were placed on them
        used = 0.0 if mem_used is None else mem_used[k]
        if cached is None:
            hr = hc = 0
        else:
            rows, cols = _as_sets(cached[k])
            hr = _covered(rows, origin[0], origin[0] + m)
            hc = _covered(cols, origin[1], origin[1] + q)

        def ok(x, d=d, hr=hr, hc=hc, used=used):
            af, bf = max(0, x - hr), max(0, x - hc)
            return (shard_cost(d, x, x, n, b, af, bf) <= T and
                    float(af * n * b + n * bf * b + x * x * b) + used <= d.mem_bytes)
        edges.append(_largest(top, g, ok) * g)
    order = sorted((k for k in range(len(devs)) if edges[k] > 0), key=lambda k: (-edges[k], k))
    band_h, col_w, owner = [], [], []
    pos = 0
    rows_left = m
    while rows_left > 0:
        if pos >= len(order):
            return None
        h = min(edges[order[pos]], rows_left)
        widths, owners = [], []
        cols_left = q
        while cols_left > 0:
            if pos >= len(order):
                return None
            k = order[pos]
            pos += 1
            r_lo, c_lo = m - rows_left, q - cols_left

            def ok(w, k=k, h=h, cols_left=cols_left, r_lo=r_lo, c_lo=c_lo):
                w = min(w, cols_left)
                return cost_at(k, r_lo, h, c_lo, w) <= T and fits_at(k, r_lo, h, c_lo, w)
            w = min(_largest(-(-cols_left // g), g, ok) * g, cols_left)
            if w == 0:
                continue
            widths.append(w)
            owners.append(k)
            cols_left -= w
        band_h.append(h)
        col_w.append(widths)
        owner.append(owners)
        rows_left -= h
    return band_h, col_w, owner


def assign(m, q, n, b, devs, granule, origin=(0, 0), cached=None, mem_used=None):
    """Returns (band_h, col_w, owner, cost): band heights (sum m), one list of
    column widths per band (each sums to q), the device of every tile, and the
    GEMM cost max_k C(alpha_k, beta_k).  Raises ValueError if no feasible
    layout exists (memory).  With `cached` / `mem_used` / `origin` this is the
    churn re-solve of Sec. 4.2: the m x q rectangle is the failed devices'
    unfinished output, `devs` the survivors, and the downlink term counts only
    rows and columns a device does not hold yet."""
    if min(m, q, n, b, granule) < 1 or not devs:
        raise ValueError("sizes must be positive and the device list non-empty")
    if (cached is None) != (mem_used is None):
        raise ValueError("cached and mem_used come together")
    t_hi = 1e-9
    found = None
    for _ in range(80):
        found = _layout(m, q, n, b, devs, granule, t_hi, origin, cached, mem_used)
        if found is not None:
            break
        t_hi *= 2.0
    if found is None:
        raise ValueError("no feasible assignment (memory capacities too small)")
    lo, hi = 0.0, t_hi
    for _ in range(64):
        mid = (lo + hi) / 2.0
        lay = _layout(m, q, n, b, devs, granule, mid, origin, cached, mem_used)
        if lay is not None:
            hi, found = mid, lay
        else:
            lo = mid
    band_h, col_w, owner = found
    cost = 0.0
    r_lo = 0
    for h, widths, owners in zip(band_h, col_w, owner):
        c_lo = 0
        for w, k in zip(widths, owners):
            if cached is None:
                c = shard_cost(devs[k], h, w, n, b)
            else:
                rows, cols = _as_sets(cached[k])
                a_lo, c0 = origin[0] + r_lo, origin[1] + c_lo
                c = shard_cost(devs[k], h, w, n, b, h - _covered(rows, a_lo, a_lo + h),
                               w - _covered(cols, c0, c0 + w))
            cost = max(cost, c)
            c_lo += w
        r_lo += h
    return band_h, col_w, owner, cost


def gemm_cost(devs, shards, n, b):
    """max_k C(alpha_k, beta_k) for shards = [(device index, alpha, beta), ...]."""
    return max((shard_cost(devs[k], a, be, n, b) for k, a, be in shards), default=0.0)
