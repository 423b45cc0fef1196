"""Host-side tests of the library (no GPU needed): the C-ABI exports every
declared symbol, and the library's task planner is byte-identical to the
oracle's on all benchmark configurations, ragged and heterogeneous plans."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2512_22142_amd as cleave
from oracle import planner
from workloads import layer_config, draw_explicit_tiling
from workloads.configs import C4_TILING_SEED

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def same_bytes(lib_tasks, oracle_tasks):
    return lib_tasks.tobytes() == oracle_tasks.tobytes()


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "cleave.h")).read()
    declared = set(re.findall(r"\b(cleave_[a-z_0-9]+)\s*\(", header))
    assert declared == set(cleave.EXPORTS)
    lib = ctypes.CDLL(cleave.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert cleave.version() == 107
    assert cleave.TASK_DTYPE.itemsize == planner.TASK_DTYPE.itemsize == 64


@pytest.mark.parametrize("args", [
    (512, 512, 512, 128, 128, 2), (300, 200, 64, 128, 128, 1), (7, 5, 6, 3, 2, 3),
    (1, 1, 1, 1, 1, 1), (1000, 777, 333, 256, 512, 8), (4096, 11008, 4096, 512, 512, 4),
    (5, 9, 7, 8, 4, 7), (130, 150, 10, 64, 64, 3),
])
def test_uniform_plan_matches_oracle_bytes(args):
    M, N, K, tm, tn, S = args
    p = cleave.plan_uniform(M, N, K, tm, tn, S, gemm_id=3)
    tasks, elems = planner.plan_uniform(M, N, K, tm, tn, S, gemm_id=3)
    assert p.num_tasks == len(tasks) and p.partial_elems == elems
    assert (p.M, p.N, p.K) == (M, N, K)
    assert p.num_tiles == len(tasks) // S
    assert same_bytes(p.tasks, tasks)


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c5"])
def test_config_plans_match_oracle_bytes(name):
    cfg = layer_config(name)
    for gid, g in enumerate(cfg.gemms):
        p = cleave.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit, gemm_id=gid)
        tasks, elems = planner.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit, gemm_id=gid)
        assert p.partial_elems == elems
        assert same_bytes(p.tasks, tasks), g.name


def test_heterogeneous_plans_match_oracle_bytes():
    cfg = layer_config("c4")
    for gid, g in enumerate(cfg.gemms):
        band_h, col_w, ks = draw_explicit_tiling(g.M, g.N, g.K, C4_TILING_SEED + gid)
        p = cleave.plan_explicit(g.M, g.N, g.K, band_h, col_w, ks, gemm_id=gid)
        tasks, elems = planner.plan_explicit(g.M, g.N, g.K, band_h, col_w, ks, gemm_id=gid)
        assert p.partial_elems == elems and p.num_tiles == len(ks)
        assert same_bytes(p.tasks, tasks), g.name
    # small odd-sized case
    p = cleave.plan_explicit(7, 9, 8, [2, 4, 1], [[3, 6], [9], [1, 1, 7]], [1, 2, 4, 8, 1, 2])
    tasks, _ = planner.plan_explicit(7, 9, 8, [2, 4, 1], [[3, 6], [9], [1, 1, 7]], [1, 2, 4, 8, 1, 2])
    assert same_bytes(p.tasks, tasks)


@pytest.mark.parametrize("args", [
    (0, 8, 8, 4, 4, 1), (8, 0, 8, 4, 4, 1), (8, 8, 0, 4, 4, 1), (8, 8, 8, 0, 4, 1),
    (8, 8, 8, 4, 0, 1), (8, 8, 8, 4, 4, 0), (8, 8, 5, 4, 4, 4), (8, 8, 4, 4, 4, 5),
    (2 ** 31, 8, 8, 4, 4, 1),
])
def test_uniform_plan_rejects_what_the_oracle_rejects(args):
    with pytest.raises(cleave.CleaveError) as e:
        cleave.plan_uniform(*args)
    assert e.value.status == -1
    if args[0] < 2 ** 31:
        with pytest.raises(planner.PlanError):
            planner.plan_uniform(*args)


@pytest.mark.parametrize("band_h,col_w,ks", [
    ([4, 3], [[8], [8]], [1, 1]),
    ([4, 4], [[8], [4, 3]], [1, 1, 1]),
    ([4, 5], [[8], [8]], [1, 1]),
    ([4, 4], [[8], [4, 5]], [1, 1, 1]),
    ([8, 0], [[8], [8]], [1, 1]),
    ([4, 4], [[8], [8, 0]], [1, 1, 1]),
    ([4, 4], [[8], [8]], [1, 9]),
])
def test_explicit_plan_rejects_bad_lists(band_h, col_w, ks):
    with pytest.raises(cleave.CleaveError):
        cleave.plan_explicit(8, 8, 8, band_h, col_w, ks)
    with pytest.raises(planner.PlanError):
        planner.plan_explicit(8, 8, 8, band_h, col_w, ks)


def test_plan_whose_indices_would_wrap_is_rejected():
    big = 2**31 - 1
    with pytest.raises(cleave.CleaveError) as e:
        cleave.plan_uniform(big, big, 64, big, big, 1)   # one tile of 2^48 sub-tiles
    assert e.value.status == -1


def test_null_arguments_are_errors_not_crashes():
    lib = ctypes.CDLL(cleave.LIB_PATH)
    lib.cleave_plan_uniform.argtypes = [ctypes.c_int64] * 5 + [ctypes.c_int32, ctypes.c_uint32, ctypes.c_void_p]
    assert lib.cleave_plan_uniform(8, 8, 8, 4, 4, 1, 0, None) == -1
    lib.cleave_plan_num_tasks.argtypes = [ctypes.c_void_p]
    lib.cleave_plan_num_tasks.restype = ctypes.c_int64
    assert lib.cleave_plan_num_tasks(None) == -1
    lib.cleave_plan_destroy.argtypes = [ctypes.c_void_p]
    lib.cleave_plan_destroy(None)
    lib.cleave_execute.argtypes = [ctypes.c_void_p] * 2 + [ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
                                   ctypes.c_int, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int,
                                   ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.cleave_execute(None, None, 0, None, 0, 0, None, 0, 0, 0, None, None) == -1
    lib.cleave_reduce.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int64, ctypes.c_int, ctypes.c_void_p]
    assert lib.cleave_reduce(None, None, None, 0, 0, None) == -1
    lib.cleave_strerror.restype = ctypes.c_char_p
    assert lib.cleave_strerror(-1) == b"invalid argument"


@pytest.mark.parametrize("args", [(20, 12, 16, 8, 8, 2, 5), (1024, 1024, 128, 512, 512, 1, 128),
                                  (7, 5, 6, 3, 2, 3, 1), (192, 192, 64, 128, 128, 1, 6)])
def test_batched_plan_matches_oracle_bytes(args):
    tasks, elems = planner.plan_batched(*args)
    p = cleave.plan_batched(*args)
    assert p.tasks.tobytes() == tasks.tobytes()
    assert p.num_tasks == len(tasks) and p.partial_elems == elems
    assert (p.M, p.N, p.K) == args[:3]


def test_batched_plan_rejects_empty_batch_and_bad_split():
    for args in [(8, 8, 8, 4, 4, 1, 0), (8, 8, 4, 4, 4, 5, 2), (0, 8, 8, 4, 4, 1, 2)]:
        with pytest.raises(cleave.CleaveError) as e:
            cleave.plan_batched(*args)
        assert e.value.status == -1


# ---- workgroup schedule of the fast kernel (host logic) -----------------------

def _loads(plan, which, grid):
    import paper_2512_22142_amd as cleave
    return cleave.schedule_loads(plan, which, grid, False), cleave.schedule_loads(plan, which, grid, True)


def test_schedule_of_equal_items_is_the_strided_one():
    import paper_2512_22142_amd as cleave
    plan = cleave.plan_uniform(4096, 4096, 4096, 512, 512, 4)      # 1024 items of 16 K steps
    strided, used = _loads(plan, 0, 256)
    assert np.array_equal(strided, used)
    assert np.all(used == 4 * (16 + 4.5))


def test_schedule_of_unequal_items_is_balanced():
    """Tiles with 1, 2, 4, 8 splits: the schedule conserves the work, beats the
    every-grid-th rule, and meets the bound of longest-first list scheduling
    (no workgroup exceeds the mean by more than one item -- the longest)."""
    import paper_2512_22142_amd as cleave
    M, N, K = 4096, 6144, 4096
    band_h = [512] * 8
    col_w = [[512] * 12 for _ in band_h]
    ks = [(1, 2, 4, 8)[(3 * i + j) % 4] for i in range(8) for j in range(12)]
    plan = cleave.plan_explicit(M, N, K, band_h, col_w, ks)
    for grid in (256, 304, 64):
        strided, used = _loads(plan, 0, grid)
        assert abs(strided.sum() - used.sum()) < 1e-9 and used.min() > 0
        longest = K / 64 + 4.5
        assert used.max() <= used.mean() + longest + 1e-9
        assert used.max() < strided.max()
        assert used.mean() / used.max() > 0.9, (grid, used.mean() / used.max())
    # fewer items than workgroups: one item each, nothing to balance
    strided, used = _loads(plan, 0, 4096)
    assert np.array_equal(strided, used)


def test_schedule_loads_argument_errors():
    import paper_2512_22142_amd as cleave
    plan = cleave.plan_uniform(512, 512, 512, 256, 256, 1)
    for which, grid in ((3, 8), (-1, 8), (0, 0)):
        with pytest.raises(cleave.CleaveError):
            cleave.schedule_loads(plan, which, grid)
