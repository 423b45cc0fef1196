"""GPU parity at the benchmark configurations' full sizes, in the launch
configuration the benchmark times (whole-plan execute + reduce per GEMM).

A full fp64 oracle GEMM is used where it takes about a second; otherwise every
GEMM of every configuration is checked by (i) the fp64 random-projection
identity over the whole of C, (ii) the full-K fp64 oracle on sampled output
tiles (always including the last, ragged tile) and (iii) the per-task fp64
oracle on sampled partial blocks -- both against the contractual Frobenius bar
and element by element against a bound derived from fp32 accumulation -- plus
the bitwise aggregation check on sampled tiles.  The whole-output,
every-element comparison at these sizes is in test_gpu_exact_full.py.
"""
import numpy as np
import pytest
import torch

import paper_2512_22142_amd as cleave
from oracle import gemm as og
from oracle import planner
from workloads import layer_config, make_gemm_operands, draw_explicit_tiling, draw_reissue
from workloads.configs import C4_TILING_SEED, C4_REISSUE_SEED

from gpu_util import TOL, assert_elementwise, block_of, elementwise_bound

pytestmark = pytest.mark.gpu

PROJECTION_BOUND = 1e-4      # a wrong 128x128 block of a 4096x11008 output reads ~1e-2


class DeviceTensors:
    """Device copies of a configuration's tensors, made on first use."""

    def __init__(self, cfg):
        self.cfg = cfg
        self.cpu = {}
        self.dev = {}

    def operands(self, g):
        A, B = make_gemm_operands(self.cfg, g, cache=self.cpu)
        for name, t in ((g.a, A), (g.b, B)):
            if name not in self.dev:
                self.dev[name] = t.cuda()
        return A, B, self.dev[g.a], self.dev[g.b]


def sample_tiles(tasks, rng, count):
    tiles = np.unique(tasks["tile_id"])
    picks = {int(tiles[-1])}                           # last tile: ragged corner if any
    while len(picks) < min(count, len(tiles)):
        picks.add(int(rng.choice(tiles)))
    return sorted(picks)


def check_gemm_sampled(g, plan, tasks, A, B, dA, dB, dtype, rng, n_tiles=2, full=False):
    partials = torch.empty(plan.partial_elems, dtype=torch.float32, device="cuda")
    C = torch.empty((g.M, g.N), dtype=torch.float32, device="cuda")
    cleave.execute(plan, dA, dB, partials, g.transA, g.transB)
    cleave.reduce(plan, partials, C)
    torch.cuda.synchronize()
    Ch = C.cpu().numpy()
    opA, opB = og.logical_operands(A, g.transA, B, g.transB)
    assert og.projection_check(opA, opB, Ch, seed=int(rng.integers(1 << 30))) < PROJECTION_BOUND, g.name
    if full:
        assert og.rel_frobenius(Ch, og.gemm(opA, opB)) <= TOL[dtype], g.name
    for tile in sample_tiles(tasks, rng, n_tiles):
        sel = tasks[tasks["tile_id"] == tile]
        t0 = sel[0]
        m0, ml, n0, nl = int(t0["m0"]), int(t0["m_len"]), int(t0["n0"]), int(t0["n_len"])
        ref = og.output_block(opA, opB, m0, ml, n0, nl)
        got = Ch[m0:m0 + ml, n0:n0 + nl]
        assert og.rel_frobenius(got, ref) <= TOL[dtype], (g.name, tile)          # the contractual bar
        rows, cols = opA[m0:m0 + ml, :], opB[:, n0:n0 + nl]
        if dtype == "bf16":
            # element by element: the S chunk sums and their S - 1 additions each round like one chunk
            bound = sum(elementwise_bound(rows, cols, int(t["k0"]), int(t["k0"]) + int(t["k_len"])) for t in sel)
            assert_elementwise(got, ref, bound + 2.0 ** -23 * len(sel) * np.abs(ref), (g.name, tile))
        # this tile's partial blocks: fetch only their slice of the buffer
        lo = int(t0["partial_off"])
        hi = lo + len(sel) * ml * nl
        seg = partials[lo:hi].cpu().numpy()
        scale = np.linalg.norm(ref) + 1e-30
        s_pick = int(rng.integers(len(sel)))
        blk = og.task_block(opA, opB, sel[s_pick])
        got_blk = seg[s_pick * ml * nl:(s_pick + 1) * ml * nl].reshape(ml, nl)
        assert np.linalg.norm(got_blk - blk) <= TOL[dtype] * scale, (g.name, tile, s_pick)
        if dtype == "bf16":
            k0 = int(sel[s_pick]["k0"])
            assert_elementwise(got_blk, blk, elementwise_bound(rows, cols, k0, k0 + int(sel[s_pick]["k_len"])),
                               (g.name, tile, s_pick))
        # aggregation of this tile, bitwise
        local = sel.copy()
        local["partial_off"] -= lo
        local["m0"] = 0
        local["n0"] = 0
        assert np.array_equal(og.reduce_partials(local, seg, ml, nl), got), (g.name, tile)
    return partials, C, opA, opB


def test_c2_gpt2_small_layer():
    cfg = layer_config("c2")
    dt = DeviceTensors(cfg)
    rng = np.random.default_rng(cfg.seed)
    for gid, g in enumerate(cfg.gemms):
        plan = cleave.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit, gemm_id=gid)
        tasks, _ = planner.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit, gemm_id=gid)
        assert plan.tasks.tobytes() == tasks.tobytes()
        A, B, dA, dB = dt.operands(g)
        check_gemm_sampled(g, plan, tasks, A, B, dA, dB, cfg.dtype, rng, n_tiles=3,
                           full=g.name in ("o.fwd", "o.dx", "o.dw"))
        print("c2", g.name, plan.num_tasks, "tasks", plan.last_kernel, flush=True)


def test_c3_llama7b_layer():
    cfg = layer_config("c3")
    dt = DeviceTensors(cfg)
    rng = np.random.default_rng(cfg.seed)
    for gid, g in enumerate(cfg.gemms):
        plan = cleave.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit, gemm_id=gid)
        tasks, _ = planner.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit, gemm_id=gid)
        assert plan.tasks.tobytes() == tasks.tobytes()
        A, B, dA, dB = dt.operands(g)
        check_gemm_sampled(g, plan, tasks, A, B, dA, dB, cfg.dtype, rng, n_tiles=2)
        print("c3", g.name, plan.num_tasks, "tasks", plan.last_kernel, flush=True)


def test_c4_heterogeneous_tiles_and_reissue():
    cfg = layer_config("c4")
    dt = DeviceTensors(cfg)
    rng = np.random.default_rng(C4_TILING_SEED)
    for gid, g in enumerate(cfg.gemms):
        band_h, col_w, ks = draw_explicit_tiling(g.M, g.N, g.K, C4_TILING_SEED + gid)
        plan = cleave.plan_explicit(g.M, g.N, g.K, band_h, col_w, ks, gemm_id=gid)
        tasks, _ = planner.plan_explicit(g.M, g.N, g.K, band_h, col_w, ks, gemm_id=gid)
        assert plan.tasks.tobytes() == tasks.tobytes()
        A, B, dA, dB = dt.operands(g)
        partials, C, opA, opB = check_gemm_sampled(g, plan, tasks, A, B, dA, dB, cfg.dtype, rng, n_tiles=3)
        # churn: 5 % of the tasks are lost and issued again, in shuffled order
        first = partials.clone()
        C_first = C.clone()
        lost = draw_reissue(plan.num_tasks, C4_REISSUE_SEED + gid, 0.05)
        for i in lost:
            off = int(tasks[i]["partial_off"])
            partials[off:off + int(tasks[i]["m_len"]) * int(tasks[i]["n_len"])] = float("nan")
        cleave.execute(plan, dA, dB, partials, g.transA, g.transB, task_ids=lost)
        torch.cuda.synchronize()
        assert torch.equal(partials.view(torch.int32), first.view(torch.int32)), g.name
        cleave.reduce(plan, partials, C)
        torch.cuda.synchronize()
        assert torch.equal(C.view(torch.int32), C_first.view(torch.int32)), g.name
        print("c4", g.name, plan.num_tasks, "tasks,", len(lost), "re-issued", flush=True)


def test_c5_llama13b_layer():
    cfg = layer_config("c5")
    dt = DeviceTensors(cfg)
    rng = np.random.default_rng(cfg.seed)
    for gid, g in enumerate(cfg.gemms):
        plan = cleave.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit, gemm_id=gid)
        tasks, _ = planner.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit, gemm_id=gid)
        assert plan.tasks.tobytes() == tasks.tobytes()
        A, B, dA, dB = dt.operands(g)
        check_gemm_sampled(g, plan, tasks, A, B, dA, dB, cfg.dtype, rng, n_tiles=2)
        print("c5", g.name, plan.num_tasks, "tasks", plan.last_kernel, flush=True)
