"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle.

Bars: task plan byte-identical (checked on the host elsewhere); C within a
relative Frobenius error of 1e-5 for fp32 inputs and 5e-3 for bf16 inputs with
fp32 accumulation; bit-exact for integer-valued inputs; re-executed tasks
bitwise identical; the aggregation bitwise equal to the oracle's fp32 left
fold of the same partials.
"""
import numpy as np
import pytest
import torch

import paper_2512_22142_amd as cleave
from oracle import gemm as og
from oracle import planner
from workloads import layer_config, make_tensor, draw_reissue
from workloads.tensors import make_matrix

from gpu_util import GpuGemm, TOL, block_of, stored

pytestmark = pytest.mark.gpu

LAYOUTS = [(0, 0), (0, 1), (1, 0), (1, 1)]


def check_against_oracle(run, opA, opB, dtype, tasks):
    """Full comparison: every partial block and the reduced C."""
    parts = run.partials_host()
    C = run.C_host()
    ref = og.gemm(opA, opB)
    err = og.rel_frobenius(C, ref)
    assert err <= TOL[dtype], err
    # partial blocks, one by one, against the oracle's per-task product
    scale = np.linalg.norm(ref) / np.sqrt(ref.size) + 1e-30
    for t in tasks:
        blk = og.task_block(opA, opB, t)
        got = block_of(parts, t)
        assert np.linalg.norm(got - blk) <= TOL[dtype] * (np.linalg.norm(blk) + scale), int(t["tile_id"])
    # aggregation: bitwise the oracle's fp32 left fold of these partials
    fold = og.reduce_partials(tasks, parts, run.plan.M, run.plan.N)
    assert np.array_equal(fold, C)
    return err


def test_c1_fp32_512_full():
    cfg = layer_config("c1")
    g = cfg.gemms[0]
    A, B = make_tensor(cfg, "a"), make_tensor(cfg, "b")
    plan = cleave.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit)
    tasks, elems = planner.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit)
    assert plan.tasks.tobytes() == tasks.tobytes() and plan.num_tasks == 32
    run = GpuGemm(plan, A, B).run()
    opA, opB = og.logical_operands(A, 0, B, 0)
    err = check_against_oracle(run, opA, opB, "f32", tasks)
    print("c1 rel Frobenius error %.3e, kernel %s" % (err, plan.last_kernel))


# (M, N, K, tile_m, tile_n, S): several tiles and a ragged tail; the first rows
# keep every size a multiple of 8 (16-byte load path), the later ones do not
# (guarded element path); 384/640-sized tiles exercise the 256-edge sub-tiling.
SHAPES = [
    (256, 256, 128, 128, 128, 2),
    (320, 200, 192, 128, 128, 3),
    (640, 520, 256, 512, 384, 2),
    (520, 776, 320, 520, 776, 1),
    (77, 45, 51, 32, 32, 2),
    (300, 259, 130, 128, 256, 4),
    (513, 270, 67, 513, 270, 1),
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("transA,transB", LAYOUTS)
@pytest.mark.parametrize("shape", SHAPES)
def test_small_shapes_all_layouts(shape, transA, transB, dtype):
    M, N, K, tm, tn, S = shape
    a = make_matrix(M * 7 + K, M, K, dtype)
    b = make_matrix(N * 5 + K + 1, K, N, dtype, std=0.5)
    A, B = stored(a, transA), stored(b, transB)
    plan = cleave.plan_uniform(M, N, K, tm, tn, S)
    tasks, _ = planner.plan_uniform(M, N, K, tm, tn, S)
    assert plan.tasks.tobytes() == tasks.tobytes()
    run = GpuGemm(plan, A, B, transA, transB).run()
    opA, opB = og.logical_operands(A, transA, B, transB)
    check_against_oracle(run, opA, opB, dtype, tasks)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("transA,transB", LAYOUTS)
def test_integer_inputs_are_bit_exact(transA, transB, dtype):
    M, N, K = 392, 328, 448
    a = make_matrix(61, M, K, dtype, integer_valued=True)
    b = make_matrix(62, K, N, dtype, integer_valued=True)
    exact = (a.to(torch.int64) @ b.to(torch.int64)).numpy().astype(np.float64)
    A, B = stored(a, transA), stored(b, transB)
    opA, opB = og.logical_operands(A, transA, B, transB)
    assert np.array_equal(og.gemm(opA, opB), exact)
    for tm, tn, S in [(128, 128, 1), (392, 328, 7), (264, 136, 4)]:
        plan = cleave.plan_uniform(M, N, K, tm, tn, S)
        run = GpuGemm(plan, A, B, transA, transB).run()
        assert np.array_equal(run.C_host().astype(np.float64), exact), (tm, tn, S)


def test_heterogeneous_plan_small():
    M, N, K = 600, 520, 384
    band_h = [128, 256, 216]
    col_w = [[256, 264], [520], [128, 128, 264]]
    ks = [1, 2, 4, 8, 2, 1]
    a = make_matrix(71, M, K, "bf16")
    b = make_matrix(72, K, N, "bf16", std=0.02)
    plan = cleave.plan_explicit(M, N, K, band_h, col_w, ks)
    tasks, _ = planner.plan_explicit(M, N, K, band_h, col_w, ks)
    assert plan.tasks.tobytes() == tasks.tobytes()
    run = GpuGemm(plan, a, b).run()
    opA, opB = og.logical_operands(a, 0, b, 0)
    check_against_oracle(run, opA, opB, "bf16", tasks)


def test_mixed_chunk_lengths_reissue_bitwise():
    """Tiles whose chunks are whole K steps of the fast kernel next to tiles whose
    chunks are not (K = 768: S = 1, 2, 4 give 768, 384, 192; S = 8 gives 96): a
    block's bits depend on its own task record only, whichever other tasks run
    in the same call and in whatever order they are listed."""
    M, N, K = 768, 768, 768
    band_h = [512, 256]
    col_w = [[256, 512], [256, 256, 256]]
    ks = [8, 1, 2, 8, 4]
    a = make_matrix(73, M, K, "bf16")
    b = make_matrix(74, K, N, "bf16", std=0.02)
    plan = cleave.plan_explicit(M, N, K, band_h, col_w, ks)
    tasks, _ = planner.plan_explicit(M, N, K, band_h, col_w, ks)
    assert plan.tasks.tobytes() == tasks.tobytes()
    run = GpuGemm(plan, a, b).run()
    opA, opB = og.logical_operands(a, 0, b, 0)
    check_against_oracle(run, opA, opB, "bf16", tasks)
    first = run.partials_host().copy()
    lost = [len(tasks) - 1, 0, 9, 8, 3, 12]            # both kinds, not in canonical order
    assert {int(tasks[i]["k_len"]) % 64 for i in lost} == {0, 32}
    poisoned = first.copy()
    for i in lost:
        block_of(poisoned, tasks[i])[:] = np.nan
    run.partials.copy_(torch.from_numpy(poisoned).cuda())
    run.execute(task_ids=lost)
    assert run.partials_host().tobytes() == first.tobytes()
    for i in (0, 8):                                     # one task alone
        run.partials.fill_(float("nan"))
        run.execute(task_ids=[i])
        assert block_of(run.partials_host(), tasks[i]).tobytes() == block_of(first, tasks[i]).tobytes()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_reissued_tasks_are_bitwise_identical(dtype):
    M, N, K = 768, 640, 512
    a = make_matrix(81, M, K, dtype)
    b = make_matrix(82, K, N, dtype, std=0.02)
    plan = cleave.plan_uniform(M, N, K, 384, 128, 4)     # both sub-tile classes
    tasks = plan.tasks
    run = GpuGemm(plan, a, b).run()
    first = run.partials_host().copy()
    C_first = run.C_host().copy()
    lost = draw_reissue(plan.num_tasks, seed=5, fraction=0.2)
    poisoned = first.copy()
    for i in lost:
        block_of(poisoned, tasks[i])[:] = np.nan
    run.partials.copy_(torch.from_numpy(poisoned).cuda())
    run.execute(task_ids=lost)
    again = run.partials_host()
    assert again.tobytes() == first.tobytes()      # re-issued blocks identical, others untouched
    assert run.reduce().C_host().tobytes() == C_first.tobytes()
    # a second full execution is bitwise identical as well
    run.partials.fill_(float("nan"))
    assert run.execute().partials_host().tobytes() == first.tobytes()


def test_execute_rejects_bad_task_ids():
    plan = cleave.plan_uniform(128, 128, 64, 64, 64, 1)
    a = make_matrix(1, 128, 64, "bf16")
    b = make_matrix(2, 64, 128, "bf16")
    run = GpuGemm(plan, a, b)
    for ids in ([4], [-1], [0, 0]):
        with pytest.raises(cleave.CleaveError):
            run.execute(task_ids=ids)
    with pytest.raises(ValueError):
        cleave.execute(plan, run.A, run.A, run.partials)


def test_reduce_single_split_is_a_copy_and_bf16_output_rounds_to_nearest_even():
    M, N = 200, 136
    plan = cleave.plan_uniform(M, N, 16, 64, 72, 1)
    tasks = plan.tasks
    rng = np.random.default_rng(3)
    parts = rng.standard_normal(plan.partial_elems).astype(np.float32)
    parts[:4] = [np.float32(1.00390625), np.float32(1.01171875), np.inf, -0.0]   # ties: to even
    d_parts = torch.from_numpy(parts).cuda()
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")
    cleave.reduce(plan, d_parts, C)
    ref = og.reduce_partials(tasks, parts, M, N)
    assert np.array_equal(C.cpu().numpy(), ref)
    Cb = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    cleave.reduce(plan, d_parts, Cb)
    assert torch.equal(Cb.cpu(), torch.from_numpy(ref).to(torch.bfloat16))
    # strided C (ldc > N) and a split count of 8, odd sizes (element path)
    plan8 = cleave.plan_uniform(37, 29, 64, 16, 16, 8)
    parts8 = (rng.standard_normal(plan8.partial_elems) * 100).astype(np.float32)
    big = torch.zeros((37, 40), dtype=torch.float32, device="cuda")
    cleave.reduce(plan8, torch.from_numpy(parts8).cuda(), big[:, :29])
    ref8 = og.reduce_partials(plan8.tasks, parts8, 37, 29)
    assert np.array_equal(big[:, :29].cpu().numpy(), ref8)
    assert float(big[:, 29:].abs().sum()) == 0.0
