"""cleave_execute_noalloc, the entry point for callers that cannot allocate:
its output against cleave_execute's, bit for bit, on calls in a row that share
the fixed work-list array (the second with a smaller subset), its size limit
and its refusal to upload."""
import numpy as np
import pytest
import torch

import paper_2512_22142_amd as cleave
from workloads import draw_reissue
from workloads.tensors import make_matrix

from gpu_util import GpuGemm

pytestmark = pytest.mark.gpu


def _poison(partials, tasks, ids):
    for i in ids:
        off = int(tasks[i]["partial_off"])
        partials[off:off + int(tasks[i]["m_len"]) * int(tasks[i]["n_len"])] = float("nan")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_noalloc_subsets_match_execute_on_consecutive_calls(dtype):
    M, N, K = 1408, 1160, 768
    a = make_matrix(301, M, K, dtype)
    b = make_matrix(302, K, N, dtype, std=0.02)
    # 384-edge tiles: both sub-tile classes, clipped sub-tiles; S = 8 gives 96-element
    # chunks (staged kernel for bf16), S = 4 gives 192 (direct kernel)
    band_h = [384, 384, 384, 256]
    col_w = [[384, 384, 392]] * 4
    ks = [4, 8, 4, 8, 4, 8, 4, 8, 4, 8, 4, 8]
    plan = cleave.plan_explicit(M, N, K, band_h, col_w, ks)
    tasks = plan.tasks
    run = GpuGemm(plan, a, b).execute()          # uploads the plan's tables
    torch.cuda.synchronize()
    ref_full = run.partials.clone()

    # whole plan through the no-allocation entry point
    out = torch.full_like(ref_full, float("nan"))
    cleave.execute_noalloc(plan, run.A, run.B, out)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int32), ref_full.view(torch.int32))

    # two subset calls in a row, the second smaller: each against cleave_execute on the same ids
    for seed, fraction in ((7, 0.6), (8, 0.15), (9, 0.02)):
        lost = draw_reissue(plan.num_tasks, seed=seed, fraction=fraction)
        want = torch.full_like(ref_full, float("nan"))
        cleave.execute(plan, run.A, run.B, want, task_ids=lost)
        got = torch.full_like(ref_full, float("nan"))
        cleave.execute_noalloc(plan, run.A, run.B, got, task_ids=lost)
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int32), want.view(torch.int32)), (seed, fraction)
        # and those blocks are the full launch's blocks, everything else untouched (still NaN)
        written = ~torch.isnan(got)
        assert torch.equal(got[written].view(torch.int32), ref_full[written].view(torch.int32))
        assert int(written.sum()) == sum(int(tasks[i]["m_len"]) * int(tasks[i]["n_len"]) for i in lost)


def test_noalloc_refuses_oversized_subsets_and_plans_not_uploaded():
    M = N = 8192
    K = 64
    plan = cleave.plan_uniform(M, N, K, 64, 64, 1)      # 16384 tasks of one work item each
    a = make_matrix(311, M, K, "bf16")
    b = make_matrix(312, K, N, "bf16")
    dA, dB = a.cuda(), b.cuda()
    partials = torch.full((plan.partial_elems,), float("nan"), dtype=torch.float32, device="cuda")
    with pytest.raises(cleave.CleaveError) as e:        # tables not on the device yet
        cleave.execute_noalloc(plan, dA, dB, partials, task_ids=[0])
    assert e.value.status == cleave.EINVAL
    plan.upload()
    cleave.execute_noalloc(plan, dA, dB, partials, task_ids=list(range(plan.num_tasks)))   # exactly the limit
    torch.cuda.synchronize()
    want = torch.empty_like(partials)
    cleave.execute(plan, dA, dB, want)
    torch.cuda.synchronize()
    assert torch.equal(partials.view(torch.int32), want.view(torch.int32))

    big = cleave.plan_uniform(M, N + 64, K, 64, 64, 1)  # 16512 tasks
    big.upload()
    b2 = make_matrix(313, K, N + 64, "bf16").cuda()
    p2 = torch.full((big.partial_elems,), float("nan"), dtype=torch.float32, device="cuda")
    with pytest.raises(cleave.CleaveError) as e:
        cleave.execute_noalloc(big, dA, b2, p2, task_ids=list(range(big.num_tasks)))
    assert e.value.status == cleave.ELIMIT
    torch.cuda.synchronize()
    assert bool(torch.isnan(p2).all())                   # nothing was enqueued
    cleave.execute_noalloc(big, dA, b2, p2, task_ids=list(range(16384)))   # within the limit again
    torch.cuda.synchronize()
    assert not bool(torch.isnan(p2[:16384 * 64 * 64]).any())
