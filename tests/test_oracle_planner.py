"""Pins for the oracle's task planner: brute-force coverage on tiny shapes, the
paper's constraints (exact cover, no redundant work, no empty task, 2mnq flop
count), closed-form task tables and hand-derived task counts."""
import itertools

import numpy as np
import pytest

from oracle import planner
from workloads import layer_config, draw_explicit_tiling


def brute_force_cover(tasks, M, N, K):
    """Counts how often every (i, j, k) triple of the GEMM is computed."""
    hits = np.zeros((M, N, K), dtype=np.int32)
    for t in tasks:
        hits[t["m0"]:t["m0"] + t["m_len"],
             t["n0"]:t["n0"] + t["n_len"],
             t["k0"]:t["k0"] + t["k_len"]] += 1
    return hits


@pytest.mark.parametrize("M,N,K,tm,tn,S", [
    (1, 1, 1, 1, 1, 1), (8, 8, 8, 4, 4, 2), (7, 5, 6, 3, 2, 3), (5, 9, 7, 8, 4, 7),
    (6, 6, 5, 6, 6, 1), (3, 4, 8, 2, 3, 4), (9, 2, 3, 4, 5, 2),
])
def test_uniform_plan_covers_every_triple_once(M, N, K, tm, tn, S):
    tasks, elems = planner.plan_uniform(M, N, K, tm, tn, S)
    assert (brute_force_cover(tasks, M, N, K) == 1).all()
    assert elems == S * M * N          # one m x q output per K-split (coverage constraint)
    assert planner.check_plan_invariants(tasks, M, N, K)


def test_explicit_plan_covers_every_triple_once():
    M, N, K = 7, 9, 8
    band_h = [2, 4, 1]
    col_w = [[3, 6], [9], [1, 1, 7]]
    ks = [1, 2, 4, 8, 1, 2]
    tasks, elems = planner.plan_explicit(M, N, K, band_h, col_w, ks)
    assert (brute_force_cover(tasks, M, N, K) == 1).all()
    assert len(tasks) == sum(ks)
    assert elems == sum(h * w * s for h, ws, sl in
                        zip(band_h, col_w, ([1, 2], [4], [8, 1, 2])) for w, s in zip(ws, sl))
    assert planner.check_plan_invariants(tasks, M, N, K)


def test_c1_task_table_closed_form():
    # 512^3 GEMM, 128x128 tiles, 2 K-splits: 32 tasks of 128 x 128 x 256.
    tasks, elems = planner.plan_uniform(512, 512, 512, 128, 128, 2)
    assert len(tasks) == 32 and elems == 2 * 512 * 512
    for i, t in enumerate(tasks):
        tile, s = divmod(i, 2)
        r, c = divmod(tile, 4)
        expect = dict(gemm_id=0, tile_id=tile, m0=128 * r, m_len=128, n0=128 * c, n_len=128,
                      k0=256 * s, k_len=256, ksplit_idx=s, ksplit_cnt=2,
                      partial_off=i * 128 * 128, flags=0)
        for key, val in expect.items():
            assert int(t[key]) == val, (i, key)


def test_ragged_tiles_are_clipped_not_padded():
    tasks, elems = planner.plan_uniform(300, 200, 64, 128, 128, 1)
    dims = [(int(t["m0"]), int(t["m_len"]), int(t["n0"]), int(t["n_len"])) for t in tasks]
    assert dims == [(0, 128, 0, 128), (0, 128, 128, 72),
                    (128, 128, 0, 128), (128, 128, 128, 72),
                    (256, 44, 0, 128), (256, 44, 128, 72)]
    assert elems == 300 * 200
    offs = [int(t["partial_off"]) for t in tasks]
    assert offs == [0, 16384, 16384 + 9216, 2 * 16384 + 9216, 2 * 16384 + 2 * 9216,
                    2 * 16384 + 2 * 9216 + 44 * 128]


def test_k_chunks_rule():
    assert planner.k_chunks(512, 2) == [(0, 256), (256, 256)]
    assert planner.k_chunks(10, 3) == [(0, 4), (4, 4), (8, 2)]     # kc = ceil(10/3) = 4
    assert planner.k_chunks(7, 7) == [(i, 1) for i in range(7)]
    with pytest.raises(planner.PlanError):
        planner.k_chunks(5, 4)       # kc = 2, chunk 3 would start at 6 >= 5: empty
    with pytest.raises(planner.PlanError):
        planner.k_chunks(4, 5)       # more splits than inner elements
    with pytest.raises(planner.PlanError):
        planner.k_chunks(4, 0)


def test_explicit_rejects_bad_edge_lists():
    with pytest.raises(planner.PlanError):
        planner.plan_explicit(8, 8, 8, [4, 3], [[8], [8]], [1, 1])       # bands sum to 7
    with pytest.raises(planner.PlanError):
        planner.plan_explicit(8, 8, 8, [4, 4], [[8], [4, 3]], [1, 1, 1])  # widths sum to 7
    with pytest.raises(planner.PlanError):
        planner.plan_explicit(8, 8, 8, [4, 4], [[8], [4, 4]], [1, 1])     # too few S
    with pytest.raises(planner.PlanError):
        planner.plan_explicit(8, 8, 8, [4, 4], [[8], [4, 4]], [1, 1, 1, 1])
    with pytest.raises(planner.PlanError):
        planner.plan_explicit(8, 8, 8, [8, 0], [[8], [8]], [1, 1])        # empty band


def test_explicit_equals_uniform_on_uniform_cuts():
    M, N, K, tm, tn, S = 300, 520, 96, 128, 256, 3
    u, ue = planner.plan_uniform(M, N, K, tm, tn, S)
    band_h = [128, 128, 44]
    col_w = [[256, 256, 8]] * 3
    e, ee = planner.plan_explicit(M, N, K, band_h, col_w, [S] * 9)
    assert ue == ee and u.tobytes() == e.tobytes()


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c5"])
def test_config_task_counts_and_flops(name, golden):
    counts = [int(v) for v in golden("task_counts.txt")[name]]
    flops = int(golden("layer_flops.txt")[name][0])
    cfg = layer_config(name)
    per_kind = {"fwd": 0, "dx": 0, "dw": 0}
    total_flops = 0
    for g in cfg.gemms:
        tasks, elems = planner.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit)
        per_kind[g.kind] += len(tasks)
        assert elems == cfg.ksplit * g.M * g.N
        vol = (tasks["m_len"].astype(np.int64) * tasks["n_len"] * tasks["k_len"]).sum()
        assert vol == g.M * g.N * g.K          # no redundant work
        total_flops += 2 * int(vol)            # 2mnq convention
        assert tasks["m_len"].min() >= 1 and tasks["n_len"].min() >= 1 and tasks["k_len"].min() >= 1
    assert [sum(per_kind.values()), per_kind["fwd"], per_kind["dx"], per_kind["dw"]] == counts
    assert total_flops == flops == cfg.flops


def test_config_plan_invariants_full_check():
    cfg = layer_config("c3")
    for g in cfg.gemms[:7:3]:
        tasks, _ = planner.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit)
        planner.check_plan_invariants(tasks, g.M, g.N, g.K)


def test_heterogeneous_draw_gives_valid_plans():
    for seed, (M, N, K) in enumerate([(4096, 11008, 4096), (4096, 4096, 11008), (1000, 777, 333)]):
        band_h, col_w, ks = draw_explicit_tiling(M, N, K, 1004 + seed)
        tasks, elems = planner.plan_explicit(M, N, K, band_h, col_w, ks)
        planner.check_plan_invariants(tasks, M, N, K)
        assert set(ks) <= {1, 2, 4, 8}
        assert elems == sum(int(t["m_len"]) * int(t["n_len"]) for t in tasks)
    # a small case is additionally brute-forced
    band_h, col_w, ks = draw_explicit_tiling(300, 260, 40, 7)
    tasks, _ = planner.plan_explicit(300, 260, 40, band_h, col_w, ks)
    assert (brute_force_cover(tasks, 300, 260, 40) == 1).all()


def test_invariant_checker_catches_planted_mistakes():
    tasks, _ = planner.plan_uniform(64, 64, 32, 32, 32, 2)
    for field, delta in [("m0", 1), ("n_len", -1), ("k0", 1), ("k_len", -1), ("partial_off", 4)]:
        bad = tasks.copy()
        bad[field][3] = int(bad[field][3]) + delta
        with pytest.raises(AssertionError):
            planner.check_plan_invariants(bad, 64, 64, 32)
    with pytest.raises(AssertionError):      # a task listed twice = redundant work
        planner.check_plan_invariants(np.concatenate([tasks, tasks[-1:]]), 64, 64, 32)


def test_batched_plan_is_the_single_plan_repeated_with_running_offsets():
    M, N, K, tm, tn, S, G = 20, 12, 16, 8, 8, 2, 5
    tasks, elems = planner.plan_batched(M, N, K, tm, tn, S, G)
    one, one_elems = planner.plan_uniform(M, N, K, tm, tn, S)
    assert elems == G * M * N * S == G * one_elems and len(tasks) == G * len(one)
    for g in range(G):
        part = tasks[g * len(one):(g + 1) * len(one)].copy()
        assert np.all(part["gemm_id"] == g)
        # each member alone is a valid plan of the single GEMM
        local = part.copy()
        local["partial_off"] -= g * one_elems
        local["gemm_id"] = 0
        assert local.tobytes() == one.tobytes()
        planner.check_plan_invariants(local, M, N, K)
    # blocks are disjoint and cover [0, elems) exactly
    sizes = tasks["m_len"].astype(np.int64) * tasks["n_len"]
    assert np.array_equal(tasks["partial_off"], np.concatenate([[0], np.cumsum(sizes)[:-1]]))
    # attention-score shape of the paper's table: 1024 x 128 x 1024 per head, K too short to split
    t, e = planner.plan_batched(1024, 1024, 128, 512, 512, 1, 128)
    assert len(t) == 128 * 4 and e == 128 * 1024 * 1024
    with pytest.raises(planner.PlanError):
        planner.plan_batched(8, 8, 8, 4, 4, 1, 0)
