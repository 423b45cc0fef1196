"""Element-by-element GPU parity at the benchmark configurations' full sizes,
in the launch configuration the benchmark times.

Integer-valued inputs (uniform in [-4, 4], exact in bf16) make every product
and every partial sum an integer below 2^24 (K * 16 <= 16384 * 16 = 2^18), so
the fp32 path has to reproduce the fp64 oracle bit for bit, whatever the
tiling, the chunking and the order of accumulation:

  c3: all 21 GEMMs -- every partial block of every task and the whole of C,
      against the full fp64 oracle (one naive GEMM per chunk of K);
  c4: all 21 GEMMs with their heterogeneous tilings -- the whole of C, sampled
      partial blocks, then 5 % of the tasks re-issued (bitwise);
  c5: GEMMs of each kind, layout and chunk length (640, 1728, 2048), ragged
      13824-wide outputs included -- full-K oracle on bands of rows across
      all columns.

These cover what a sampled Frobenius comparison cannot: isolated wrong
elements anywhere in the output, in workgroups that run many work items in a
row.
"""
import numpy as np
import pytest
import torch

import paper_2512_22142_amd as cleave
from oracle import gemm as og
from oracle import planner
from workloads import layer_config, make_gemm_operands, draw_explicit_tiling, draw_reissue
from workloads.configs import C4_TILING_SEED, C4_REISSUE_SEED

from gpu_util import block_of

pytestmark = pytest.mark.gpu

# exact C of c3's GEMMs with integer-valued inputs (c4 multiplies the same tensors)
_C3_EXACT = {}


class IntegerTensors:
    def __init__(self, cfg):
        self.cfg, self.cpu, self.dev = cfg, {}, {}

    def operands(self, g):
        A, B = make_gemm_operands(self.cfg, g, cache=self.cpu, integer_valued=True)
        for name, t in ((g.a, A), (g.b, B)):
            if name not in self.dev:
                self.dev[name] = t.cuda()
        return A, B, self.dev[g.a], self.dev[g.b]


def run_gemm(plan, g, dA, dB):
    partials = torch.empty(plan.partial_elems, dtype=torch.float32, device="cuda")
    C = torch.empty((g.M, g.N), dtype=torch.float32, device="cuda")
    cleave.execute(plan, dA, dB, partials, g.transA, g.transB)
    cleave.reduce(plan, partials, C)
    torch.cuda.synchronize()
    return partials, C


def test_c3_integer_inputs_every_partial_block_and_all_of_C_exact():
    cfg = layer_config("c3")
    it = IntegerTensors(cfg)
    for gid, g in enumerate(cfg.gemms):
        plan = cleave.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit, gemm_id=gid)
        tasks, _ = planner.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit, gemm_id=gid)
        assert plan.tasks.tobytes() == tasks.tobytes()
        A, B, dA, dB = it.operands(g)
        partials, C = run_gemm(plan, g, dA, dB)
        parts = partials.cpu().numpy()
        opA, opB = og.logical_operands(A, g.transA, B, g.transB)
        total = np.zeros((g.M, g.N), dtype=np.float64)
        for s in range(cfg.ksplit):
            sel = tasks[tasks["ksplit_idx"] == s]
            k0, k1 = int(sel[0]["k0"]), int(sel[0]["k0"]) + int(sel[0]["k_len"])
            assert np.all(sel["k0"] == k0) and np.all(sel["k_len"] == k1 - k0)
            ref = og.gemm(opA, opB, k0, k1)                      # chunk s of the whole GEMM
            for t in sel:
                m0, ml, n0, nl = int(t["m0"]), int(t["m_len"]), int(t["n0"]), int(t["n_len"])
                assert np.array_equal(block_of(parts, t), ref[m0:m0 + ml, n0:n0 + nl]), \
                    (g.name, int(t["tile_id"]), s)
            total += ref
        assert np.abs(total).max() < 2 ** 24
        assert np.array_equal(C.cpu().numpy(), total), g.name
        _C3_EXACT[g.name] = total.astype(np.float32)
        print("c3 exact", g.name, plan.num_tasks, "blocks", plan.last_kernel, flush=True)
        del parts, partials, C, total


def test_c4_integer_inputs_all_gemms_exact_then_reissue():
    cfg = layer_config("c4")
    it = IntegerTensors(cfg)
    rng = np.random.default_rng(C4_TILING_SEED)
    for gid, g in enumerate(cfg.gemms):
        band_h, col_w, ks = draw_explicit_tiling(g.M, g.N, g.K, C4_TILING_SEED + gid)
        plan = cleave.plan_explicit(g.M, g.N, g.K, band_h, col_w, ks, gemm_id=gid)
        tasks, _ = planner.plan_explicit(g.M, g.N, g.K, band_h, col_w, ks, gemm_id=gid)
        assert plan.tasks.tobytes() == tasks.tobytes()
        A, B, dA, dB = it.operands(g)
        partials, C = run_gemm(plan, g, dA, dB)
        opA, opB = og.logical_operands(A, g.transA, B, g.transB)
        exact = _C3_EXACT.get(g.name)
        if exact is None:                                   # this test run on its own
            exact = og.gemm(opA, opB)
        assert np.array_equal(C.cpu().numpy(), exact), g.name
        # partial blocks of sampled tiles (all of their chunks), exact
        tiles = np.unique(tasks["tile_id"])
        for tile in {int(tiles[-1]), *(int(x) for x in rng.choice(tiles, 3))}:
            for t in tasks[tasks["tile_id"] == tile]:
                off, cnt = int(t["partial_off"]), int(t["m_len"]) * int(t["n_len"])
                got = partials[off:off + cnt].cpu().numpy().reshape(int(t["m_len"]), int(t["n_len"]))
                assert np.array_equal(got, og.task_block(opA, opB, t)), (g.name, tile, int(t["ksplit_idx"]))
        # churn: 5 % of the tasks are lost and issued again, in shuffled order
        first, C_first = partials.clone(), C.clone()
        lost = draw_reissue(plan.num_tasks, C4_REISSUE_SEED + gid, 0.05)
        for i in lost:
            off = int(tasks[i]["partial_off"])
            partials[off:off + int(tasks[i]["m_len"]) * int(tasks[i]["n_len"])] = float("nan")
        cleave.execute(plan, dA, dB, partials, g.transA, g.transB, task_ids=lost)
        cleave.reduce(plan, partials, C)
        torch.cuda.synchronize()
        assert torch.equal(partials.view(torch.int32), first.view(torch.int32)), g.name
        assert torch.equal(C.view(torch.int32), C_first.view(torch.int32)), g.name
        print("c4 exact", g.name, plan.num_tasks, "tasks,", len(lost), "re-issued", flush=True)
    _C3_EXACT.clear()


# c5 GEMMs by name: forward NN, dX NT, dW TN; chunk lengths K/8 = 640 (K = 5120),
# 1728 (K = 13824), 2048 (K = 16384); gate/up outputs are 13824 wide (ragged last tile)
C5_EXACT_GEMMS = ("q.fwd", "gate.fwd", "down.fwd", "q.dx", "gate.dx", "down.dx", "q.dw", "up.dw", "down.dw")
C5_BAND_ROWS = 192          # rows per checked band: crosses no tile edge by itself ...
C5_BANDS = 3                # ... so the bands are placed across tile edges, and at the end


def test_c5_integer_inputs_row_bands_exact():
    cfg = layer_config("c5")
    it = IntegerTensors(cfg)
    rng = np.random.default_rng(cfg.seed)
    seen_chunks = set()
    for gid, g in enumerate(cfg.gemms):
        if g.name not in C5_EXACT_GEMMS:
            continue
        plan = cleave.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit, gemm_id=gid)
        tasks, _ = planner.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit, gemm_id=gid)
        assert plan.tasks.tobytes() == tasks.tobytes()
        seen_chunks.add(int(tasks[0]["k_len"]))
        A, B, dA, dB = it.operands(g)
        partials, C = run_gemm(plan, g, dA, dB)
        opA, opB = og.logical_operands(A, g.transA, B, g.transB)
        # bands of rows over all columns: one across a tile edge, one random, the last rows
        edge = cfg.tile_m * int(rng.integers(1, g.M // cfg.tile_m)) - C5_BAND_ROWS // 2
        starts = [edge, int(rng.integers(0, g.M - C5_BAND_ROWS)), g.M - C5_BAND_ROWS][:C5_BANDS]
        for r0 in starts:
            ref = og.gemm(opA[r0:r0 + C5_BAND_ROWS, :], opB)
            got = C[r0:r0 + C5_BAND_ROWS, :].cpu().numpy()
            assert np.array_equal(got, ref), (g.name, r0)
        # every chunk's partial block of one sampled tile, and of the last (ragged) tile
        tiles = np.unique(tasks["tile_id"])
        for tile in {int(tiles[-1]), int(rng.choice(tiles))}:
            for t in tasks[tasks["tile_id"] == tile][::3]:
                off, cnt = int(t["partial_off"]), int(t["m_len"]) * int(t["n_len"])
                got = partials[off:off + cnt].cpu().numpy().reshape(int(t["m_len"]), int(t["n_len"]))
                assert np.array_equal(got, og.task_block(opA, opB, t)), (g.name, tile, int(t["ksplit_idx"]))
        print("c5 exact", g.name, plan.num_tasks, "tasks", plan.last_kernel, flush=True)
        del partials, C, opA, opB
    assert seen_chunks == {640, 1728, 2048}
