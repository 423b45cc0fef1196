"""The shard assignment of the library (C ABI, host only) against definitions
that do not share its construction (Sec. 4.1 cost model and constraints,
Appendix "Communication Efficiency: Heterogeneous", Eq. 18):

  * validity, checked on the library's own output: the shards cover the m x q
    output exactly once (painted cell by cell), one shard per device, no empty
    shard (zero-task constraint), every shard fits its device (memory
    constraint), and the reported cost is max_k C(alpha_k, beta_k) recomputed
    from the cost equations;
  * lower bounds no assignment can beat: total work over total compute rate
    and the cheapest single-element shard (Eq. 18), and each device's fixed
    latency;
  * quality: the exact optimum over ALL guillotine layouts on a coarse granule
    with the best assignment of distinct devices to tiles, found by exhaustive
    enumeration of layouts and a bottleneck matching per layout -- no
    bisection, no device ordering, nothing of the heuristic.

The cost equations themselves are pinned by hand values in
test_oracle_scheduler.py; only `shard_cost` / `shard_fits` of the oracle are
used here."""
import itertools

import numpy as np
import pytest

import paper_2512_22142_amd as cleave
from oracle import scheduler as sc
from workloads import draw_fleet


def lib_and_model(fleet):
    return [cleave.Device(*d) for d in fleet], [sc.Device(*d) for d in fleet]


def check_library_layout(m, q, n, b, model, res):
    band_h, col_w, owner, cost = res
    paint = np.zeros((m, q), dtype=np.int16)
    used, worst, r = [], 0.0, 0
    for h, widths, owners in zip(band_h, col_w, owner):
        c = 0
        for w, k in zip(widths, owners):
            assert h >= 1 and w >= 1                                   # zero-task constraint
            assert sc.shard_fits(model[k], h, w, n, b)                 # memory constraint
            paint[r:r + h, c:c + w] += 1
            worst = max(worst, sc.shard_cost(model[k], h, w, n, b))
            used.append(k)
            c += w
        r += h
    assert np.all(paint == 1)                                          # coverage: exactly once
    assert len(used) == len(set(used))                                 # one shard per device
    assert cost == worst                                               # GEMM cost = max over devices
    return used


def lower_bound(m, q, n, b, model):
    """Eq. 18 for one GEMM (work 2 m q n, divisible down to one output
    element) and the latency floor of the cheapest device."""
    work = 2.0 * m * q * n
    total_rate = sum(d.flops for d in model)
    single = min(sc.shard_cost(d, 1, 1, n, b) for d in model)
    return max(work / total_rate, single)


def compositions(total):
    if total == 0:
        yield ()
        return
    for first in range(1, total + 1):
        for rest in compositions(total - first):
            yield (first,) + rest


def bottleneck_assignment(cost):
    """min over injective maps tile -> device of the max cost; cost[t][k] = inf
    where the shard does not fit.  Threshold search over the distinct cost
    values with augmenting-path matching."""
    n_t, n_k = len(cost), len(cost[0])
    if n_t > n_k:
        return float("inf")

    def feasible(limit):
        match = [-1] * n_k

        def augment(t, seen):
            for k in range(n_k):
                if cost[t][k] <= limit and not seen[k]:
                    seen[k] = True
                    if match[k] < 0 or augment(match[k], seen):
                        match[k] = t
                        return True
            return False
        return all(augment(t, [False] * n_k) for t in range(n_t))
    values = sorted({c for row in cost for c in row if c != float("inf")})
    lo, hi = 0, len(values) - 1
    if not values or not feasible(values[hi]):
        return float("inf")
    while lo < hi:
        mid = (lo + hi) // 2
        if feasible(values[mid]):
            hi = mid
        else:
            lo = mid + 1
    return values[lo]


def exact_guillotine_optimum(m, q, n, b, model, g):
    best = float("inf")
    col_patterns = list(compositions(q // g))
    for bands in compositions(m // g):
        if len(bands) > len(model):
            continue
        for cols in itertools.product(col_patterns, repeat=len(bands)):
            if sum(len(c) for c in cols) > len(model):
                continue
            tiles = [(h * g, w * g) for h, ws in zip(bands, cols) for w in ws]
            cost = [[sc.shard_cost(d, h, w, n, b) if sc.shard_fits(d, h, w, n, b) else float("inf")
                     for d in model] for h, w in tiles]
            best = min(best, bottleneck_assignment(cost))
    return best


def test_bottleneck_assignment_by_hand():
    inf = float("inf")
    assert bottleneck_assignment([[3.0, 1.0], [2.0, 5.0]]) == 2.0        # tile0->dev1, tile1->dev0
    assert bottleneck_assignment([[3.0, 1.0], [4.0, 5.0]]) == 4.0        # tile1 must take dev0 (4), tile0 dev1
    assert bottleneck_assignment([[1.0, inf], [2.0, inf]]) == inf         # two tiles, one usable device
    assert bottleneck_assignment([[7.0, 9.0, 8.0]]) == 7.0
    assert bottleneck_assignment([[1.0], [1.0]]) == inf


RATIOS = []


@pytest.mark.parametrize("seed", range(30))
def test_library_against_the_exact_guillotine_optimum(seed):
    rng = np.random.default_rng(500 + seed)
    g, b = 16, 2
    m, q = g * int(rng.integers(2, 6)), g * int(rng.integers(2, 6))
    n = int(rng.choice([64, 256, 1024]))
    k = int(rng.integers(3, 8))
    fleet = draw_fleet(k, 900 + seed)
    if seed % 3 == 0:
        # tighten the memories so that the constraint shapes the optimum
        fleet = [d[:5] + (float((2 * g) * n * b * 2 + (2 * g) * (2 * g) * b),) for d in fleet]
    lib, model = lib_and_model(fleet)
    opt = exact_guillotine_optimum(m, q, n, b, model, g)
    if opt == float("inf"):
        with pytest.raises(cleave.CleaveError):
            cleave.assign(m, q, n, b, lib, g)
        return
    res = cleave.assign(m, q, n, b, lib, g)
    check_library_layout(m, q, n, b, model, res)
    assert res[3] >= opt * (1 - 1e-12)                  # the layout is one of the enumerated ones
    assert res[3] >= lower_bound(m, q, n, b, model) * (1 - 1e-12)
    RATIOS.append(res[3] / opt)
    assert res[3] <= 1.15 * opt, (res[3], opt)          # observed over these instances: 1.000 ... 1.073 (median 1.000)


@pytest.mark.parametrize("m,q,n,k,g,seed", [(4096, 4096, 4096, 32, 64, 1), (4096, 11008, 4096, 100, 64, 2),
                                            (1000, 777, 333, 7, 16, 3), (131072, 4096, 4096, 512, 128, 4)])
def test_library_layout_is_valid_and_above_the_lower_bounds_at_scale(m, q, n, k, g, seed):
    lib, model = lib_and_model(draw_fleet(k, 40 + seed))
    res = cleave.assign(m, q, n, 2, lib, g)
    if m * q <= 1 << 26:
        check_library_layout(m, q, n, 2, model, res)
    else:                                               # too large to paint: areas and sums instead
        assert sum(res[0]) == m and all(sum(w) == q for w in res[1])
        owners = [d for row in res[2] for d in row]
        assert len(owners) == len(set(owners))
        assert sum(h * w for h, ws in zip(res[0], res[1]) for w in ws) == m * q
    assert res[3] >= lower_bound(m, q, n, 2, model)


def test_observed_ratios_to_the_optimum():
    # runs after the parametrised cases above; documents what the bound of 1.4 rests on
    if RATIOS:
        print("heuristic / exact guillotine optimum: min %.3f  median %.3f  max %.3f over %d instances"
              % (min(RATIOS), float(np.median(RATIOS)), max(RATIOS), len(RATIOS)))


# ---- churn re-solve with general cache sets (Sec. 4.2: binary matrices R_s, C_s) ----

def random_sets(rng, n_dev, extent, max_iv):
    """Per device a sorted list of disjoint intervals inside [0, extent)."""
    out = []
    for _ in range(n_dev):
        cuts = np.sort(rng.choice(extent + 1, size=2 * int(rng.integers(0, max_iv + 1)), replace=False))
        out.append([(int(cuts[2 * i]), int(cuts[2 * i + 1])) for i in range(len(cuts) // 2)])
    return out


@pytest.mark.parametrize("seed", range(6))
def test_resolve_with_cache_sets_against_the_binary_cache_matrices(seed):
    rng = np.random.default_rng(700 + seed)
    M, Q, n, b, g = 1024, 768, 512, 2, 32
    k = int(rng.integers(4, 12))
    fleet = draw_fleet(k, 60 + seed)
    lib, model = lib_and_model(fleet)
    row_sets = random_sets(rng, k, M, 4)
    col_sets = random_sets(rng, k, Q, 4)
    # the paper's matrices: R[k, i] = 1 iff device k holds row i of A, C[k, j] likewise for columns of B
    R = np.zeros((k, M), dtype=bool)
    C = np.zeros((k, Q), dtype=bool)
    for d in range(k):
        for lo, hi in row_sets[d]:
            R[d, lo:hi] = True
        for lo, hi in col_sets[d]:
            C[d, lo:hi] = True
    r0, c0 = g * int(rng.integers(0, 8)), g * int(rng.integers(0, 6))
    m, q = g * int(rng.integers(4, 17)), g * int(rng.integers(4, 13))
    m, q = min(m, M - r0), min(q, Q - c0)
    used = [float(rng.integers(0, 1 << 20)) for _ in range(k)]
    cached = [(row_sets[d], col_sets[d]) for d in range(k)]
    got = cleave.assign(m, q, n, b, lib, g, origin=(r0, c0), cached=cached, mem_used=used)
    band_h, col_w, owner, cost = got
    paint = np.zeros((m, q), dtype=np.int16)
    worst, r, seen = 0.0, 0, []
    for h, widths, owners in zip(band_h, col_w, owner):
        c = 0
        for w, d in zip(widths, owners):
            paint[r:r + h, c:c + w] += 1
            a_hat = h - int(R[d, r0 + r:r0 + r + h].sum())       # rows still to fetch
            b_hat = w - int(C[d, c0 + c:c0 + c + w].sum())       # columns still to fetch
            worst = max(worst, sc.shard_cost(model[d], h, w, n, b, a_hat, b_hat))
            assert float(a_hat * n * b + n * b_hat * b + h * w * b) + used[d] <= model[d].mem_bytes
            seen.append(d)
            c += w
        r += h
    assert np.all(paint == 1) and len(seen) == len(set(seen))
    assert cost == worst
    # the oracle's construction gives the same layout (transcription check of the interval arithmetic)
    ref = sc.assign(m, q, n, b, model, g, origin=(r0, c0), cached=cached, mem_used=used)
    assert got == ref
    # caches can only help: the blind re-solve is no faster
    blind = cleave.assign(m, q, n, b, lib, g, origin=(r0, c0), cached=[([], [])] * k, mem_used=used)
    assert cost <= blind[3]


def test_single_interval_sets_equal_the_interval_form_and_bad_sets_are_rejected():
    lib, _ = lib_and_model(draw_fleet(6, 5))
    one = [(10, 200, 30, 300), (0, 0, 0, 0), (100, 400, 0, 50), (5, 6, 7, 8), (0, 512, 0, 384), (300, 301, 383, 384)]
    sets = [([(a, b_)], [(c, d)]) for a, b_, c, d in one]
    used = [0.0] * 6
    assert cleave.assign(512, 384, 256, 2, lib, 64, cached=one, mem_used=used) == \
        cleave.assign(512, 384, 256, 2, lib, 64, cached=sets, mem_used=used)
    for bad in ([(5, 3)], [(0, 10), (5, 20)], [(10, 20), (0, 5)], [(-1, 4)]):
        with pytest.raises(cleave.CleaveError):
            cleave.assign(512, 384, 256, 2, lib, 64, cached=[(bad, [])] + [([], [])] * 5, mem_used=used)
