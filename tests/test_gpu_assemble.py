"""GPU parity of cleave_execute_assemble (plans without K-splits write their
blocks straight into C): against the fp64 oracle within the usual bars, and bit
for bit against cleave_execute + cleave_reduce, whose values it must equal."""
import numpy as np
import pytest
import torch

import paper_2512_22142_amd as cleave
from oracle import gemm as og
from oracle import planner
from workloads.tensors import make_matrix

from gpu_util import TOL, stored

pytestmark = pytest.mark.gpu

CASES = [
    # dtype, M, N, K, tile_m, tile_n, transA, transB
    ("bf16", 640, 392, 256, 256, 256, 0, 0), ("bf16", 640, 392, 256, 256, 256, 0, 1),
    ("bf16", 512, 768, 128, 512, 512, 1, 0), ("bf16", 300, 200, 72, 128, 128, 0, 0),
    ("bf16", 37, 29, 50, 16, 8, 1, 1), ("f32", 256, 384, 192, 128, 128, 0, 0), ("f32", 130, 150, 10, 64, 64, 0, 1),
]


@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("dtype,M,N,K,tm,tn,transA,transB", CASES)
def test_assemble_equals_execute_plus_reduce_and_the_oracle(dtype, M, N, K, tm, tn, transA, transB, out_dtype):
    A = stored(make_matrix(301, M, K, dtype), transA)
    B = stored(make_matrix(302, K, N, dtype, std=0.02), transB)
    plan = cleave.plan_uniform(M, N, K, tm, tn, 1)
    dA, dB = A.cuda(), B.cuda()
    wide = torch.full((M, N + 24), float("nan"), dtype=out_dtype, device="cuda")
    C = wide[:, :N]                                     # leading dimension > N
    cleave.execute_assemble(plan, dA, dB, C, transA, transB)
    parts = torch.empty(plan.partial_elems, dtype=torch.float32, device="cuda")
    C2 = torch.empty((M, N), dtype=out_dtype, device="cuda")
    cleave.execute(plan, dA, dB, parts, transA, transB)
    cleave.reduce(plan, parts, C2)
    torch.cuda.synchronize()
    assert torch.equal(C.contiguous().view(torch.int16 if out_dtype == torch.bfloat16 else torch.int32),
                       C2.view(torch.int16 if out_dtype == torch.bfloat16 else torch.int32))
    assert bool(torch.isnan(wide[:, N:].float()).all())  # nothing written beside C
    opA, opB = og.logical_operands(A, transA, B, transB)
    bar = TOL[dtype] if out_dtype == torch.float32 else 5e-3
    assert og.rel_frobenius(C.float().cpu().numpy(), og.gemm(opA, opB)) <= bar


@pytest.mark.parametrize("pad,shift", [(24, 0), (25, 0), (24, 1), (25, 1)])
def test_assemble_bf16_output_alignment_cases(pad, shift):
    """bf16 C with an even / odd leading dimension and a 4-byte / 2-byte aligned
    origin: the two-element and the one-element store paths give the same bits."""
    M, N, K = 384, 320, 128
    A, B = make_matrix(311, M, K, "bf16"), make_matrix(312, K, N, "bf16", std=0.02)
    plan = cleave.plan_uniform(M, N, K, 256, 256, 1)
    dA, dB = A.cuda(), B.cuda()
    ld = N + pad
    flat = torch.full((M * ld + 2,), float("nan"), dtype=torch.bfloat16, device="cuda")
    wide = flat[shift:shift + M * ld].view(M, ld)
    C = wide[:, :N]
    cleave.execute_assemble(plan, dA, dB, C)
    parts = torch.empty(plan.partial_elems, dtype=torch.float32, device="cuda")
    C2 = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    cleave.execute(plan, dA, dB, parts)
    cleave.reduce(plan, parts, C2)
    torch.cuda.synchronize()
    assert torch.equal(C.contiguous().view(torch.int16), C2.view(torch.int16))
    assert bool(torch.isnan(wide[:, N:].float()).all())
    assert bool(torch.isnan(flat[:shift].float()).all()) and bool(torch.isnan(flat[shift + M * ld:].float()).all())


def test_assemble_subset_writes_only_its_tiles():
    M, N, K = 512, 384, 128
    A, B = make_matrix(303, M, K, "bf16"), make_matrix(304, K, N, "bf16", std=0.02)
    plan = cleave.plan_uniform(M, N, K, 128, 128, 1)
    tasks = plan.tasks
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    ids = [1, 5, 10]
    cleave.execute_assemble(plan, A.cuda(), B.cuda(), C, task_ids=ids)
    torch.cuda.synchronize()
    Ch = C.cpu().numpy()
    opA, opB = og.logical_operands(A, 0, B, 0)
    written = np.zeros((M, N), dtype=bool)
    for i in ids:
        t = tasks[i]
        m0, ml, n0, nl = int(t["m0"]), int(t["m_len"]), int(t["n0"]), int(t["n_len"])
        written[m0:m0 + ml, n0:n0 + nl] = True
        ref = og.output_block(opA, opB, m0, ml, n0, nl)
        assert og.rel_frobenius(Ch[m0:m0 + ml, n0:n0 + nl], ref) <= TOL["bf16"]
    assert np.isnan(Ch[~written]).all() and not np.isnan(Ch[written]).any()


def test_assemble_batched_scores_equal_the_two_call_path():
    n_seq, H, s_len, d = 2, 4, 512, 128
    G = n_seq * H
    Q = make_matrix(305, n_seq * s_len, H * d, "bf16")
    Kt = make_matrix(306, n_seq * s_len, H * d, "bf16")
    ld = H * d
    plan = cleave.plan_batched(s_len, s_len, d, 256, 256, 1, G)
    dQ, dK = Q.cuda(), Kt.cuda()
    P = torch.full((G * s_len, s_len), float("nan"), dtype=torch.bfloat16, device="cuda")
    cleave.execute_assemble(plan, dQ, dK, P, 0, 1, (s_len * ld, d), (s_len * ld, d),
                            (H * s_len * s_len, s_len * s_len), H)
    parts = torch.empty(plan.partial_elems, dtype=torch.float32, device="cuda")
    P2 = torch.empty_like(P)
    cleave.execute_batched(plan, dQ, (s_len * ld, d), dK, (s_len * ld, d), H, parts, 0, 1)
    cleave.reduce_batched(plan, parts, P2, (H * s_len * s_len, s_len * s_len), H)
    torch.cuda.synchronize()
    assert torch.equal(P.view(torch.int16), P2.view(torch.int16))
    Ph = P.float().cpu().numpy()
    Qw, Kw = og.widen(Q), og.widen(Kt)
    for g in (0, 3, G - 1):
        a = np.ascontiguousarray(og.batch_view(Qw, g, H, s_len * ld, d, s_len, d))
        b = np.ascontiguousarray(og.batch_view(Kw, g, H, s_len * ld, d, s_len, d).T)
        assert og.rel_frobenius(Ph[g * s_len:(g + 1) * s_len], og.gemm(a, b)) <= 5e-3


def test_assemble_rejects_k_splits_and_stray_strides():
    A = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda")
    C = torch.zeros(64, 64, device="cuda")
    with pytest.raises(cleave.CleaveError):
        cleave.execute_assemble(cleave.plan_uniform(64, 64, 64, 32, 32, 2), A, A, C)
    with pytest.raises(cleave.CleaveError):
        cleave.execute_assemble(cleave.plan_uniform(64, 64, 64, 32, 32, 1), A, A, C, a_strides=(8, 0))
    with pytest.raises(cleave.CleaveError):
        cleave.execute_assemble(cleave.plan_batched(64, 64, 64, 32, 32, 1, 2), A, A, C, n_inner=0)
