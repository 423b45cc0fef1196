"""GPU parity of the fused check + aggregation (cleave_verify_reduce through
the C ABI): lhs / rhs / scale / accept against the fp64 oracle of the check, C
against the oracle's fixed-order fold; and against the two separate calls:
rhs, scale and C the same bits, accept the same flags, lhs within the rounding
of a different summation order (the fused pass sums shorter runs of rows).

Partial blocks are synthetic as in the tests of the check alone: the oracle's
fp64 blocks rounded to fp32, some corrupted on the CPU, or blocks written by
cleave_execute where the two GPU paths are compared with each other.
"""
import numpy as np
import pytest
import torch

import paper_2512_22142_amd as cleave
from oracle import gemm as og
from oracle import planner
from oracle import verify as ov
from workloads import draw_explicit_tiling
from workloads.tensors import make_matrix, make_probe_vectors

from gpu_util import stored
from test_gpu_verify import LAYOUTS, SHAPES, compare, lhs_size, oracle_partials

pytestmark = pytest.mark.gpu


def gpu_verify_reduce(plan, A, B, transA, transB, partials, r, s, tol, out_dtype=torch.float32, C=None):
    n = plan.num_tasks
    out = {k: torch.full((n,), float("nan"), dtype=torch.float64, device="cuda") for k in ("lhs", "rhs", "scale")}
    accept = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    if C is None:
        C = torch.full((plan.M, plan.N), float("nan"), dtype=out_dtype, device="cuda")
    parts = partials if torch.is_tensor(partials) else torch.from_numpy(partials).cuda()
    cleave.verify_reduce(plan, A.cuda(), B.cuda(), parts, r.cuda(), s.cuda(), tol, accept, C,
                         out["lhs"], out["rhs"], out["scale"], transA=transA, transB=transB)
    torch.cuda.synchronize()
    return (out["lhs"].cpu().numpy(), out["rhs"].cpu().numpy(), out["scale"].cpu().numpy(),
            accept.cpu().numpy()), C


def separate_calls(plan, A, B, transA, transB, parts, r, s, tol, out_dtype=torch.float32):
    n = plan.num_tasks
    out = {k: torch.full((n,), float("nan"), dtype=torch.float64, device="cuda") for k in ("lhs", "rhs", "scale")}
    accept = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    C = torch.full((plan.M, plan.N), float("nan"), dtype=out_dtype, device="cuda")
    cleave.verify(plan, A.cuda(), B.cuda(), parts, r.cuda(), s.cuda(), tol, accept, out["lhs"], out["rhs"],
                  out["scale"], transA=transA, transB=transB)
    cleave.reduce(plan, parts, C)
    torch.cuda.synchronize()
    return (out["lhs"].cpu().numpy(), out["rhs"].cpu().numpy(), out["scale"].cpu().numpy(),
            accept.cpu().numpy()), C


def same_as_separate(got, sep, sizes):
    lhs, rhs, scale, accept = got
    lhs2, rhs2, scale2, accept2 = sep
    return (np.array_equal(rhs.view(np.uint64), rhs2.view(np.uint64)) and
            np.array_equal(scale.view(np.uint64), scale2.view(np.uint64)) and
            np.array_equal(accept, accept2) and np.all(np.abs(lhs - lhs2) <= 1e-12 * sizes + 1e-300))


def expect_fold(tasks, parts, M, N, out_dtype):
    ref = og.reduce_partials(tasks, parts, M, N)                      # fp32 left fold
    if out_dtype == torch.bfloat16:
        return torch.from_numpy(ref).to(torch.bfloat16).float().numpy()   # nearest-even, as the library rounds
    return ref


@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("transA,transB", LAYOUTS)
@pytest.mark.parametrize("M,N,K,tm,tn,S", SHAPES)
def test_fused_pass_matches_both_oracles(M, N, K, tm, tn, S, transA, transB, dtype, out_dtype):
    A_log = make_matrix(31 + M, M, K, dtype)
    B_log = make_matrix(32 + N, K, N, dtype, std=0.02)
    A, B = stored(A_log, transA), stored(B_log, transB)
    r, s = make_probe_vectors(33 + K, M, N)
    plan = cleave.plan_uniform(M, N, K, tm, tn, S)
    tasks, elems = planner.plan_uniform(M, N, K, tm, tn, S)
    opA, opB = og.logical_operands(A, transA, B, transB)
    bad = list(range(1, len(tasks), 3))
    parts = oracle_partials(tasks, opA, opB, elems, corrupt=bad)
    ref = ov.verify_tasks(tasks, opA, opB, parts, r.numpy(), s.numpy(), 1e-6)
    got, C = gpu_verify_reduce(plan, A, B, transA, transB, parts, r, s, 1e-6, out_dtype)
    compare(tasks, got, ref, lhs_size(tasks, parts, r.numpy(), s.numpy()))
    assert set(np.flatnonzero(got[3] == 0)) == set(bad)
    assert np.array_equal(C.float().cpu().numpy(), expect_fold(tasks, parts, M, N, out_dtype))
    # and the same bits as the two separate calls
    sep, C2 = separate_calls(plan, A, B, transA, transB, torch.from_numpy(parts).cuda(), r, s, 1e-6, out_dtype)
    assert same_as_separate(got, sep, lhs_size(tasks, parts, r.numpy(), s.numpy()))
    assert torch.equal(C, C2)


def test_fused_pass_every_split_count_of_a_heterogeneous_tiling():
    """Tiles with 1 ... 8 splits in one plan: every instantiation of the fused item."""
    M, N, K = 1536, 1280, 840          # 840 = lcm(1..8): every split count divides it
    band_h = [256, 384, 128, 512, 256]
    col_w = [[512, 256, 512], [384, 896], [1280], [128, 640, 512], [256, 256, 256, 512]]
    ks = [1, 2, 3, 4, 5, 6, 7, 8, 3, 5, 7, 2, 6]
    plan = cleave.plan_explicit(M, N, K, band_h, col_w, ks)
    tasks, elems = planner.plan_explicit(M, N, K, band_h, col_w, ks)
    assert plan.tasks.tobytes() == tasks.tobytes()
    assert sorted(set(int(t["ksplit_cnt"]) for t in tasks)) == list(range(1, 9))
    A = make_matrix(51, M, K)
    B = make_matrix(52, K, N, std=0.02)
    r, s = make_probe_vectors(53, M, N, kind="sign")     # +-1: a changed entry always shows
    opA, opB = og.logical_operands(A, 0, B, 0)
    bad = list(range(0, len(tasks), 5))
    parts = oracle_partials(tasks, opA, opB, elems, corrupt=bad)
    ref = ov.verify_tasks(tasks, opA, opB, parts, r.numpy(), s.numpy(), 1e-6)
    got, C = gpu_verify_reduce(plan, A, B, 0, 0, parts, r, s, 1e-6)
    compare(tasks, got, ref, lhs_size(tasks, parts, r.numpy(), s.numpy()))
    assert set(np.flatnonzero(got[3] == 0)) == set(bad)
    assert np.array_equal(C.cpu().numpy(), og.reduce_partials(tasks, parts, M, N))
    sep, C2 = separate_calls(plan, A, B, 0, 0, torch.from_numpy(parts).cuda(), r, s, 1e-6)
    assert same_as_separate(got, sep, lhs_size(tasks, parts, r.numpy(), s.numpy()))
    assert torch.equal(C, C2)


def test_fused_pass_drawn_heterogeneous_tiling():
    M, N, K = 1536, 1280, 512
    band_h, col_w, ks = draw_explicit_tiling(M, N, K, seed=77)
    plan = cleave.plan_explicit(M, N, K, band_h, col_w, ks)
    tasks, elems = planner.plan_explicit(M, N, K, band_h, col_w, ks)
    A = make_matrix(54, M, K)
    B = make_matrix(55, K, N, std=0.02)
    r, s = make_probe_vectors(56, M, N)
    opA, opB = og.logical_operands(A, 0, B, 0)
    parts = oracle_partials(tasks, opA, opB, elems, corrupt=[2])
    ref = ov.verify_tasks(tasks, opA, opB, parts, r.numpy(), s.numpy(), 1e-6)
    got, C = gpu_verify_reduce(plan, A, B, 0, 0, parts, r, s, 1e-6)
    compare(tasks, got, ref, lhs_size(tasks, parts, r.numpy(), s.numpy()))
    assert np.array_equal(C.cpu().numpy(), og.reduce_partials(tasks, parts, M, N))


def test_more_splits_than_the_fused_pass_carries():
    """16 splits per tile: the call runs the two passes one after the other; same results."""
    M, N, K, S = 256, 384, 1024, 16
    A = make_matrix(57, M, K)
    B = make_matrix(58, K, N, std=0.02)
    r, s = make_probe_vectors(59, M, N)
    plan = cleave.plan_uniform(M, N, K, 128, 128, S)
    tasks, elems = planner.plan_uniform(M, N, K, 128, 128, S)
    opA, opB = og.logical_operands(A, 0, B, 0)
    parts = oracle_partials(tasks, opA, opB, elems, corrupt=[3, 40])
    ref = ov.verify_tasks(tasks, opA, opB, parts, r.numpy(), s.numpy(), 1e-6)
    got, C = gpu_verify_reduce(plan, A, B, 0, 0, parts, r, s, 1e-6)
    compare(tasks, got, ref, lhs_size(tasks, parts, r.numpy(), s.numpy()))
    assert set(np.flatnonzero(got[3] == 0)) == {3, 40}
    assert np.array_equal(C.cpu().numpy(), og.reduce_partials(tasks, parts, M, N))


def test_fused_pass_is_exact_on_integer_inputs():
    M, N, K, tm, tn, S = 384, 264, 256, 128, 88, 4
    A = make_matrix(41, M, K, "bf16", integer_valued=True)
    B = make_matrix(42, K, N, "bf16", integer_valued=True)
    r, s = make_probe_vectors(43, M, N, kind="sign")
    plan = cleave.plan_uniform(M, N, K, tm, tn, S)
    tasks, elems = planner.plan_uniform(M, N, K, tm, tn, S)
    opA, opB = og.logical_operands(A, 0, B, 0)
    parts = og.execute_tasks(tasks, opA, opB, elems).astype(np.float32)
    ref = ov.verify_tasks(tasks, opA, opB, parts, r.numpy(), s.numpy(), 0.0)
    (lhs, rhs, scale, accept), C = gpu_verify_reduce(plan, A, B, 0, 0, parts, r, s, 0.0)
    assert np.array_equal(lhs, ref[0]) and np.array_equal(rhs, ref[1]) and np.array_equal(scale, ref[2])
    assert np.array_equal(lhs, rhs) and accept.all()
    assert np.array_equal(C.cpu().numpy().astype(np.float64), og.gemm(opA, opB))


@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0)])
def test_fused_pass_at_the_benchmark_size_equals_the_separate_calls(transA, transB):
    """A 7B-shaped GEMM (4096 x 11008 x 4096, 512-tiles, 4 splits; blocks written
    by cleave_execute, two of them overwritten): the fused pass agrees with
    cleave_verify and gives the bits of cleave_reduce; honest blocks pass, the others do not."""
    M, N, K = (4096, 11008, 4096) if (transA, transB) == (0, 0) else (4096, 4096, 4096)
    A = stored(make_matrix(61, M, K), transA).cuda()
    B = stored(make_matrix(62, K, N, std=0.02), transB).cuda()
    r, s = make_probe_vectors(63, M, N, kind="sign")     # +-1: a changed entry always shows
    plan = cleave.plan_uniform(M, N, K, 512, 512, 4)
    parts = torch.empty(plan.partial_elems, dtype=torch.float32, device="cuda")
    cleave.execute(plan, A, B, parts, transA, transB)
    bad = [5, plan.num_tasks - 2]
    for i in bad:
        off = int(plan.tasks[i]["partial_off"])
        parts[off + 1000] += 500.0
    got, C = gpu_verify_reduce(plan, A, B, transA, transB, parts, r, s, 1e-6)
    sep, C2 = separate_calls(plan, A, B, transA, transB, parts, r, s, 1e-6)
    # lhs sums |r_i P_ij s_j| <= sum |P_ij| for +-1 probes
    sizes = np.array([float(torch.abs(parts[int(t["partial_off"]):int(t["partial_off"]) + int(t["m_len"]) * int(t["n_len"])]).sum())
                      for t in plan.tasks])
    assert same_as_separate(got, sep, sizes)
    assert torch.equal(C, C2)
    assert set(np.flatnonzero(got[3] == 0)) == set(bad)


def test_fused_pass_argument_errors():
    plan = cleave.plan_uniform(64, 64, 64, 32, 32, 2)
    A = make_matrix(1, 64, 64).cuda()
    B = make_matrix(2, 64, 64).cuda()
    parts = torch.zeros(plan.partial_elems, device="cuda")
    r, s = (v.cuda() for v in make_probe_vectors(3, 64, 64))
    accept = torch.zeros(plan.num_tasks, dtype=torch.int32, device="cuda")
    C = torch.zeros(64, 64, device="cuda")
    with pytest.raises(cleave.CleaveError):
        cleave.verify_reduce(plan, A, B, parts, r, s, -1.0, accept, C)        # negative tolerance
    batched = cleave.plan_batched(64, 64, 64, 32, 32, 1, 2)
    with pytest.raises((cleave.CleaveError, ValueError)):
        cleave.verify_reduce(batched, A, B, parts, r, s, 1e-6, accept, C)     # plain plans only
