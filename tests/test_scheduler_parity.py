"""Host-side parity of the cost model and the shard assignment (C ABI, no GPU)
against the oracle: costs bit-equal, layouts identical, and the layout feeds
cleave_plan_explicit to the same task bytes."""
import time

import numpy as np
import pytest

import paper_2512_22142_amd as cleave
from oracle import planner
from oracle import scheduler as sc
from workloads import draw_fleet


def both(fleet):
    return [cleave.Device(*d) for d in fleet], [sc.Device(*d) for d in fleet]


def test_shard_cost_and_fit_are_bit_equal():
    rng = np.random.default_rng(5)
    lib, ora = both(draw_fleet(50, 11))
    for _ in range(2000):
        k = int(rng.integers(50))
        a, be = int(rng.integers(1, 5000)), int(rng.integers(1, 5000))
        n, b = int(rng.integers(1, 20000)), int(rng.choice([1, 2, 4]))
        af, bf = int(rng.integers(0, a + 1)), int(rng.integers(0, be + 1))
        assert cleave.shard_cost(lib[k], a, be, n, b) == sc.shard_cost(ora[k], a, be, n, b)
        assert cleave.shard_cost(lib[k], a, be, n, b, af, bf) == sc.shard_cost(ora[k], a, be, n, b, af, bf)
        assert cleave.shard_fits(lib[k], a, be, n, b) == sc.shard_fits(ora[k], a, be, n, b)
    assert cleave.shard_cost(lib[0], 0, 0, 64, 2) == 0.0
    for bad in [(0, 3), (3, 0), (-1, 2)]:
        with pytest.raises(cleave.CleaveError):
            cleave.shard_cost(lib[0], bad[0], bad[1], 64, 2)


# the paper's GEMM shapes at batch 128 x sequence 1024 (Sec. 3.1 table), smaller
# ones, and ragged ones; (m, q, n, devices, granule)
CASES = [
    (131072, 4096, 4096, 512, 128), (131072, 11008, 4096, 1024, 128), (4096, 4096, 4096, 32, 64),
    (4096, 11008, 4096, 100, 64), (1000, 777, 333, 7, 16), (64, 64, 64, 1, 64), (300, 200, 50, 40, 8),
]


@pytest.mark.parametrize("m,q,n,k,g", CASES)
def test_assignment_is_identical_to_the_oracles(m, q, n, k, g):
    lib, ora = both(draw_fleet(k, 100 + k))
    t0 = time.perf_counter()
    got = cleave.assign(m, q, n, 2, lib, g)
    dt = time.perf_counter() - t0
    ref = sc.assign(m, q, n, 2, ora, g)
    assert got[0] == ref[0] and got[1] == ref[1] and got[2] == ref[2]
    assert got[3] == ref[3]
    tiles = sum(len(w) for w in got[1])
    plan = cleave.plan_explicit(m, q, n, got[0], got[1], [1] * tiles)
    tasks, _ = planner.plan_explicit(m, q, n, ref[0], ref[1], [1] * tiles)
    assert plan.tasks.tobytes() == tasks.tobytes()
    planner.check_plan_invariants(tasks, m, q, n)
    print("assign %dx%dx%d over %d devices: %d shards, cost %.3f s, solved in %.1f ms" % (m, q, n, k, tiles, got[3], dt * 1e3))


def test_assignment_rejects_bad_input_and_infeasible_memory():
    lib, _ = both(draw_fleet(4, 1))
    with pytest.raises(cleave.CleaveError):
        cleave.assign(0, 8, 8, 2, lib, 8)
    with pytest.raises(cleave.CleaveError):
        cleave.assign(8, 8, 8, 2, lib, 0)
    tiny = [cleave.Device(1e6, 1e6, 0.0, 0.0, 1e12, 10.0)]
    with pytest.raises(cleave.CleaveError):
        cleave.assign(64, 64, 64, 2, tiny, 8)
    bad = [cleave.Device(0.0, 1e6, 0.0, 0.0, 1e12, 1e9)]
    with pytest.raises(cleave.CleaveError):
        cleave.assign(64, 64, 64, 2, bad, 8)


@pytest.mark.parametrize("m,q,n,k,g,seed", [(2048, 1536, 1024, 12, 64, 77), (4096, 4096, 4096, 40, 64, 5),
                                            (1000, 777, 333, 9, 16, 9), (131072, 4096, 4096, 256, 128, 21)])
def test_churn_resolve_is_identical_to_the_oracles(m, q, n, k, g, seed):
    """Cold start, failure of the device with the largest shard, re-solve over the
    survivors with their caches: layouts and costs equal the oracle's."""
    fleet = draw_fleet(k, seed)
    lib, ora = both(fleet)
    band_h, col_w, owner, _ = sc.assign(m, q, n, 2, ora, g)
    rects, r = {}, 0
    for h, widths, owners in zip(band_h, col_w, owner):
        c = 0
        for w, dev in zip(widths, owners):
            rects[dev] = (r, r + h, c, c + w)
            c += w
        r += h
    failed = max(rects, key=lambda d: (rects[d][1] - rects[d][0]) * (rects[d][3] - rects[d][2]))
    r0, r1, c0, c1 = rects[failed]
    alive = [d for d in range(k) if d != failed]
    cached = [rects.get(d, (0, 0, 0, 0)) for d in alive]
    used = [0.0 if d not in rects else float(((rects[d][1] - rects[d][0]) + (rects[d][3] - rects[d][2])) * n * 2 +
                                             (rects[d][1] - rects[d][0]) * (rects[d][3] - rects[d][2]) * 2)
            for d in alive]
    ref = sc.assign(r1 - r0, c1 - c0, n, 2, [ora[d] for d in alive], g, origin=(r0, c0), cached=cached, mem_used=used)
    got = cleave.assign(r1 - r0, c1 - c0, n, 2, [lib[d] for d in alive], g, origin=(r0, c0), cached=cached,
                        mem_used=used)
    assert got[0] == ref[0] and got[1] == ref[1] and got[2] == ref[2] and got[3] == ref[3]


def test_resolve_rejects_bad_caches():
    lib, _ = both(draw_fleet(2, 1))
    with pytest.raises(cleave.CleaveError):
        cleave.assign(64, 64, 64, 2, lib, 8, cached=[(0, 0, 0, 0)], mem_used=[0.0, 0.0])
    with pytest.raises(cleave.CleaveError):
        cleave.assign(64, 64, 64, 2, lib, 8, cached=[(5, 2, 0, 0), (0, 0, 0, 0)], mem_used=[0.0, 0.0])
    with pytest.raises(cleave.CleaveError):
        cleave.assign(64, 64, 64, 2, lib, 8, cached=[(0, 0, 0, 0)] * 2, mem_used=[-1.0, 0.0])
