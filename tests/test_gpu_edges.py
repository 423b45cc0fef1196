"""Edge cases of the execute / reduce path against the fp64 oracle: leading
dimensions beyond the fast path's 32-bit in-tile offsets, padded and
misaligned operand views, one-element problems, a single task larger than any
workgroup tile, a non-default stream."""
import numpy as np
import pytest
import torch

import paper_2512_22142_amd as cleave
from oracle import gemm as og
from oracle import planner
from workloads.tensors import make_matrix

from gpu_util import TOL, stored

pytestmark = pytest.mark.gpu


def run_and_check(A, B, transA, transB, plan_args, dtype, dA=None, dB=None, stream=None):
    M, N, K = plan_args[:3]
    plan = cleave.plan_uniform(*plan_args)
    tasks, elems = planner.plan_uniform(*plan_args)
    assert plan.tasks.tobytes() == tasks.tobytes()
    dA = A.cuda() if dA is None else dA
    dB = B.cuda() if dB is None else dB
    parts = torch.full((elems,), float("nan"), dtype=torch.float32, device="cuda")
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()          # the fills ran on the default stream
    cleave.execute(plan, dA, dB, parts, transA, transB, stream=stream)
    cleave.reduce(plan, parts, C, stream=stream)
    torch.cuda.synchronize()
    opA, opB = og.logical_operands(A, transA, B, transB)
    ref = og.gemm(opA, opB)
    Ch = C.cpu().numpy()
    assert not np.isnan(Ch).any()
    err = og.rel_frobenius(Ch, ref)
    assert err <= TOL[dtype], err
    assert np.array_equal(og.reduce_partials(tasks, parts.cpu().numpy(), M, N), Ch)
    return plan


@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0)])
def test_rows_longer_than_the_fast_paths_offset_range(transA, transB):
    """K-contiguous rows of more than 4 MiB: in-tile byte offsets no longer fit
    32 bits, the library must take the guarded path and still be right."""
    M, N, K = 16, 24, (1 << 21) + 192
    A = stored(make_matrix(201, M, K, "bf16", std=0.05), transA)
    B = stored(make_matrix(202, K, N, "bf16", std=0.05), transB)
    plan = run_and_check(A, B, transA, transB, (M, N, K, 16, 16, 2), "bf16")
    if not transA or transB:
        assert "direct" not in plan.last_kernel


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_padded_leading_dimensions_and_misaligned_bases(dtype):
    M, N, K = 320, 264, 256
    A = make_matrix(203, M, K, dtype)
    B = make_matrix(204, K, N, dtype, std=0.02)
    # padded rows: views into wider allocations (leading dimension > row length)
    Aw = torch.zeros(M, K + 40, dtype=A.dtype, device="cuda")
    Bw = torch.zeros(K, N + 24, dtype=B.dtype, device="cuda")
    Aw[:, :K] = A.cuda()
    Bw[:, :N] = B.cuda()
    run_and_check(A, B, 0, 0, (M, N, K, 128, 128, 2), dtype, dA=Aw[:, :K], dB=Bw[:, :N])
    # bases that are element-aligned only: views that start one element into a row
    Ao = torch.zeros(M, K + 8, dtype=A.dtype, device="cuda")
    Bo = torch.zeros(K, N + 8, dtype=B.dtype, device="cuda")
    Ao[:, 1:K + 1] = A.cuda()
    Bo[:, 1:N + 1] = B.cuda()
    run_and_check(A, B, 0, 0, (M, N, K, 128, 128, 2), dtype, dA=Ao[:, 1:K + 1], dB=Bo[:, 1:N + 1])


@pytest.mark.parametrize("args", [(1, 1, 1, 1, 1, 1), (1, 1, 1, 512, 512, 1), (3, 2, 5, 8, 8, 5), (1, 700, 9, 1, 256, 3)])
def test_tiny_problems(args):
    M, N, K = args[:3]
    A = make_matrix(205, M, K, "f32")
    B = make_matrix(206, K, N, "f32")
    run_and_check(A, B, 0, 0, args, "f32")


def test_one_task_much_larger_than_a_workgroup_tile():
    M, N, K = 2048, 1536, 512
    A = make_matrix(207, M, K, "bf16")
    B = stored(make_matrix(208, K, N, "bf16", std=0.02), 1)
    plan = run_and_check(A, B, 0, 1, (M, N, K, 4096, 4096, 1), "bf16")     # one tile, one task
    assert plan.num_tasks == 1


def test_work_on_a_side_stream():
    M, N, K = 512, 512, 512
    A = make_matrix(209, M, K, "bf16")
    B = make_matrix(210, K, N, "bf16", std=0.02)
    side = torch.cuda.Stream()
    dA, dB = A.cuda(), B.cuda()
    torch.cuda.synchronize()
    run_and_check(A, B, 0, 0, (M, N, K, 256, 256, 2), "bf16", dA=dA, dB=dB, stream=side)


def test_execute_and_reduce_replay_from_a_hip_graph():
    """The full-plan calls allocate nothing and record no memset nodes: captured
    once, every replay reproduces the eager result bit for bit."""
    M, N, K = 1024, 768, 512
    A = make_matrix(211, M, K, "bf16").cuda()
    B = make_matrix(212, K, N, "bf16", std=0.02).cuda()
    plan = cleave.plan_uniform(M, N, K, 256, 256, 2)
    parts = torch.empty(plan.partial_elems, dtype=torch.float32, device="cuda")
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")
    cleave.execute(plan, A, B, parts)          # eager: also uploads tables and sets kernel attributes
    cleave.reduce(plan, parts, C)
    torch.cuda.synchronize()
    eager = C.clone()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        cleave.execute(plan, A, B, parts)
        cleave.reduce(plan, parts, C)
    for replay in range(3):
        parts.fill_(float("nan"))
        C.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(C.view(torch.int32), eager.view(torch.int32)), replay
        # eager work of the program between replays
        cleave.execute(plan, A, B, parts)
        torch.cuda.synchronize()


def test_both_tile_classes_and_unequal_items_on_a_caller_stream_and_from_a_hip_graph():
    """A tiling with 512-wide and 128-wide tiles and 1, 2 or 4 splits: a full
    execute call launches both tile classes, each with a balanced workgroup
    schedule.  The reduce enqueued right behind it reads finished blocks --
    on the default stream, on a caller stream, and replayed from a graph."""
    M, N, K = 2560, 2304, 1024
    band_h = [512, 128, 512, 128, 512, 128, 512, 128]
    col_w = [[512, 128, 512, 128, 512, 512] for _ in band_h]
    ks = [(1, 2, 4)[(i + j) % 3] for i in range(len(band_h)) for j in range(6)]
    plan = cleave.plan_explicit(M, N, K, band_h, col_w, ks)
    tasks, elems = planner.plan_explicit(M, N, K, band_h, col_w, ks)
    assert plan.tasks.tobytes() == tasks.tobytes()
    A_cpu = make_matrix(221, M, K, "bf16", integer_valued=True)
    B_cpu = make_matrix(222, K, N, "bf16", integer_valued=True)
    A, B = A_cpu.cuda(), B_cpu.cuda()
    opA, opB = og.logical_operands(A_cpu, 0, B_cpu, 0)
    ref = og.gemm(opA, opB)
    parts = torch.full((elems,), float("nan"), dtype=torch.float32, device="cuda")
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    cleave.execute(plan, A, B, parts)
    cleave.reduce(plan, parts, C)
    torch.cuda.synchronize()
    assert np.array_equal(C.cpu().numpy().astype(np.float64), ref)
    # a caller stream of its own
    side = torch.cuda.Stream()
    for _ in range(3):
        parts.fill_(float("nan"))
        C.fill_(float("nan"))
        torch.cuda.synchronize()
        cleave.execute(plan, A, B, parts, stream=side)
        cleave.reduce(plan, parts, C, stream=side)
        torch.cuda.synchronize()
        assert np.array_equal(C.cpu().numpy().astype(np.float64), ref)
    # captured once, replayed
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        cleave.execute(plan, A, B, parts)
        cleave.reduce(plan, parts, C)
    for replay in range(3):
        parts.fill_(float("nan"))
        C.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(C.cpu().numpy().astype(np.float64), ref), replay
        cleave.execute(plan, A, B, parts)      # eager work of the program between replays
        torch.cuda.synchronize()
