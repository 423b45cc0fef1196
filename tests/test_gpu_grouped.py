"""GPU parity of the grouped form (the same-shape GEMMs of one DAG level in one
launch, one pointer per member; Sec. 4.1): every member against the fp64
oracle within the usual bars, and bit for bit against the single-GEMM calls on
the same member, whose blocks a grouped launch must reproduce."""
import numpy as np
import pytest
import torch

import paper_2512_22142_amd as cleave
from oracle import gemm as og
from oracle import planner
from workloads.tensors import make_matrix

from gpu_util import TOL, stored

pytestmark = pytest.mark.gpu


def run_group(dtype, M, N, K, tile, S, transA, transB, n, shared_a, out_dtype=torch.float32):
    """n members; with shared_a all of them read one stored A (the projections of
    a level share their input)."""
    As = [stored(make_matrix(500 + (0 if shared_a else g), M, K, dtype), transA) for g in range(n)]
    Bs = [stored(make_matrix(520 + g, K, N, dtype, std=0.02), transB) for g in range(n)]
    dA0 = As[0].cuda()
    dAs = [dA0 if shared_a else As[g].cuda() for g in range(n)]
    dBs = [b.cuda() for b in Bs]
    plan = cleave.plan_batched(M, N, K, tile, tile, S, n)
    parts = torch.full((plan.partial_elems,), float("nan"), dtype=torch.float32, device="cuda")
    Cs = [torch.full((M, N), float("nan"), dtype=out_dtype, device="cuda") for _ in range(n)]
    cleave.execute_grouped(plan, dAs, dBs, parts, transA, transB)
    cleave.reduce_grouped(plan, parts, Cs)
    torch.cuda.synchronize()
    return plan, As, Bs, dAs, dBs, parts, Cs


@pytest.mark.parametrize("dtype,M,N,K,tile,S,transA,transB,n,shared_a", [
    ("bf16", 512, 384, 256, 256, 2, 0, 0, 3, True),     # small members: one XCD each
    ("bf16", 2048, 2048, 256, 512, 2, 0, 0, 3, True),   # 128 large items per member
    ("bf16", 4096, 4096, 128, 512, 1, 0, 1, 2, False),  # 256 items per member: spread over the XCDs
    ("bf16", 4096, 2048, 128, 512, 2, 1, 0, 4, True),   # weight gradients of a level, shared X
    ("bf16", 300, 200, 72, 128, 1, 0, 1, 2, False),     # ragged, guarded path
    ("f32", 256, 384, 96, 128, 2, 0, 0, 3, True),
])
def test_grouped_equals_single_calls_and_the_oracle(dtype, M, N, K, tile, S, transA, transB, n, shared_a):
    plan, As, Bs, dAs, dBs, parts, Cs = run_group(dtype, M, N, K, tile, S, transA, transB, n, shared_a)
    tasks, elems = planner.plan_batched(M, N, K, tile, tile, S, n)
    assert plan.tasks.tobytes() == tasks.tobytes() and plan.partial_elems == elems
    single = cleave.plan_uniform(M, N, K, tile, tile, S)
    per = single.partial_elems
    assert per * n == plan.partial_elems
    p1 = torch.empty(per, dtype=torch.float32, device="cuda")
    C1 = torch.empty((M, N), dtype=torch.float32, device="cuda")
    for g in range(n):
        cleave.execute(single, dAs[g], dBs[g], p1, transA, transB)
        cleave.reduce(single, p1, C1)
        torch.cuda.synchronize()
        assert torch.equal(parts[g * per:(g + 1) * per].view(torch.int32), p1.view(torch.int32)), g
        assert torch.equal(Cs[g].view(torch.int32), C1.view(torch.int32)), g
        opA, opB = og.logical_operands(As[g], transA, Bs[g], transB)
        assert og.rel_frobenius(Cs[g].cpu().numpy(), og.gemm(opA, opB)) <= TOL[dtype], g


def test_grouped_members_at_unaligned_offsets_and_bf16_output():
    """Member pointers 8 bytes (not 16) apart from a common buffer: the guarded
    load path; bf16 results equal the rounded fp32 ones."""
    M, N, K, n = 256, 256, 128, 2
    A = make_matrix(540, M, K, "bf16")
    Bs = [make_matrix(541 + g, K, N, "bf16", std=0.02) for g in range(n)]
    dA = A.cuda()
    flat = torch.zeros(n * K * N + 4 * n, dtype=torch.bfloat16, device="cuda")
    dBs = []
    for g in range(n):
        off = g * (K * N + 4)                     # second member starts 8 bytes off a 16-byte boundary
        view = flat[off:off + K * N].view(K, N)
        view.copy_(Bs[g])
        dBs.append(view)
    plan = cleave.plan_batched(M, N, K, 128, 128, 2, n)
    parts = torch.empty(plan.partial_elems, dtype=torch.float32, device="cuda")
    Cf = [torch.empty((M, N), dtype=torch.float32, device="cuda") for _ in range(n)]
    Cb = [torch.empty((M, N), dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    cleave.execute_grouped(plan, [dA] * n, dBs, parts)
    cleave.reduce_grouped(plan, parts, Cf)
    cleave.reduce_grouped(plan, parts, Cb)
    torch.cuda.synchronize()
    for g in range(n):
        opA, opB = og.logical_operands(A, 0, Bs[g], 0)
        assert og.rel_frobenius(Cf[g].cpu().numpy(), og.gemm(opA, opB)) <= TOL["bf16"]
        assert torch.equal(Cb[g], Cf[g].to(torch.bfloat16))


def test_grouped_subset_writes_only_its_blocks():
    M, N, K, n = 512, 512, 128, 3
    A = make_matrix(550, M, K, "bf16")
    Bs = [make_matrix(551 + g, K, N, "bf16", std=0.02) for g in range(n)]
    dA, dBs = A.cuda(), [b.cuda() for b in Bs]
    plan = cleave.plan_batched(M, N, K, 256, 256, 2, n)
    tasks = plan.tasks
    full = torch.empty(plan.partial_elems, dtype=torch.float32, device="cuda")
    cleave.execute_grouped(plan, [dA] * n, dBs, full)
    parts = torch.full((plan.partial_elems,), float("nan"), dtype=torch.float32, device="cuda")
    ids = [1, len(tasks) - 1, len(tasks) // 2, 6]
    cleave.execute_grouped(plan, [dA] * n, dBs, parts, task_ids=ids)
    torch.cuda.synchronize()
    ph, fh = parts.cpu().numpy(), full.cpu().numpy()
    written = np.zeros(plan.partial_elems, dtype=bool)
    for i in ids:
        t = tasks[i]
        lo = int(t["partial_off"])
        written[lo:lo + int(t["m_len"]) * int(t["n_len"])] = True
    assert np.isnan(ph[~written]).all()
    assert ph[written].view(np.int32).tobytes() == fh[written].view(np.int32).tobytes()


def test_grouped_rejects_what_it_cannot_run():
    A = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda")
    C = torch.zeros(64, 64, device="cuda")
    parts = torch.zeros(64 * 64 * 16, device="cuda")
    plain = cleave.plan_uniform(64, 64, 64, 32, 32, 1)
    with pytest.raises(cleave.CleaveError):
        cleave.execute_grouped(plain, [A], [A], parts)
    with pytest.raises(cleave.CleaveError):
        cleave.reduce_grouped(plain, parts, [C])
    big = cleave.plan_batched(64, 64, 64, 32, 32, 1, 9)              # more members than a group holds
    with pytest.raises(cleave.CleaveError):
        cleave.execute_grouped(big, [A] * 9, [A] * 9, parts)
    two = cleave.plan_batched(64, 64, 64, 32, 32, 1, 2)
    with pytest.raises(cleave.CleaveError):
        cleave.execute_grouped(two, [A] * 3, [A] * 3, parts)         # one pointer per member, no more, no fewer
    with pytest.raises(cleave.CleaveError):
        cleave.reduce_grouped(two, parts, [C])
    wide = torch.zeros(64, 96, dtype=torch.bfloat16, device="cuda")[:, :64]
    with pytest.raises(ValueError):
        cleave.execute_grouped(two, [A, wide], [A, A], parts)        # members must share the leading dimension
