"""Seeded sweep over small random problems: sizes with and without the fast
paths' divisibility, uniform and guillotine plans with a K-split per tile, all
storage forms, both input types.  Each case: plan bytes against the oracle's
planner, C against the fp64 oracle within the usual bars, and a re-issued third
of the tasks bit for bit."""
import numpy as np
import pytest
import torch

import paper_2512_22142_amd as cleave
from oracle import gemm as og
from oracle import planner
from workloads.tensors import make_matrix

from gpu_util import TOL, GpuGemm, stored

pytestmark = pytest.mark.gpu


def cut(rng, total, choices):
    out, left = [], total
    while left > 0:
        e = min(int(rng.choice(choices)), left)
        out.append(e)
        left -= e
    return out


def valid_split(rng, K):
    S = int(rng.choice([1, 2, 3, 4, 8]))
    kc = -(-K // S)
    return S if (S - 1) * kc < K else 1


@pytest.mark.parametrize("seed", range(6))
def test_random_problems(seed):
    rng = np.random.default_rng(9000 + seed)
    for case in range(10):
        dtype = "bf16" if rng.random() < 0.75 else "f32"
        mult = 8 if rng.random() < 0.7 else 1
        M, N, K = (int(rng.integers(1, 70)) * mult for _ in range(3))
        transA, transB = int(rng.integers(0, 2)), int(rng.integers(0, 2))
        a = make_matrix(seed * 100 + case, M, K, dtype)
        b = make_matrix(seed * 100 + case + 50, K, N, dtype, std=0.05)
        if rng.random() < 0.5:
            tm, tn = int(rng.choice([16, 64, 128, 256, 384])), int(rng.choice([8, 64, 128, 256, 320]))
            S = valid_split(rng, K)
            plan = cleave.plan_uniform(M, N, K, tm, tn, S)
            tasks, _ = planner.plan_uniform(M, N, K, tm, tn, S)
        else:
            band_h = cut(rng, M, [128, 256, 384] if mult == 8 else [100, 257, 130])
            col_w = [cut(rng, N, [128, 256, 512] if mult == 8 else [99, 200, 129]) for _ in band_h]
            ks = [valid_split(rng, K) for row in col_w for _ in row]
            plan = cleave.plan_explicit(M, N, K, band_h, col_w, ks)
            tasks, _ = planner.plan_explicit(M, N, K, band_h, col_w, ks)
        label = (seed, case, dtype, M, N, K, transA, transB)
        assert plan.tasks.tobytes() == tasks.tobytes(), label
        A, B = stored(a, transA), stored(b, transB)
        run = GpuGemm(plan, A, B, transA, transB)
        run.partials.fill_(float("nan"))
        run.run()
        opA, opB = og.logical_operands(A, transA, B, transB)
        ref = og.gemm(opA, opB)
        C = run.C_host()
        assert not np.isnan(C).any(), label
        if np.linalg.norm(ref) > 0:
            assert og.rel_frobenius(C, ref) <= TOL[dtype], label
        first = run.partials_host().copy()
        ids = rng.permutation(plan.num_tasks)[:max(1, plan.num_tasks // 3)]
        run.execute(task_ids=ids)
        assert run.partials_host().tobytes() == first.tobytes(), label
