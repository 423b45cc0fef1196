"""GPU parity of the batched form (many equal-shaped GEMMs in one task list,
operands as strided zero-copy views) against the fp64 oracle, member by member.
Layouts are those of the attention products of a transformer layer (Sec. 3.1):
scores = Q K^T per (sequence, head) from token-major Q and K, and P V from
per-member contiguous P and token-major V.  Same bars as the single-GEMM tests.
"""
import numpy as np
import pytest
import torch

import paper_2512_22142_amd as cleave
from oracle import gemm as og
from oracle import planner
from workloads.tensors import make_matrix

from gpu_util import TOL

pytestmark = pytest.mark.gpu


def member_operands(Q, K, g, H, s_len, d):
    """fp64 logical operands of score GEMM g: op(A) = Q_g (s x d), op(B) = K_g^T (d x s)."""
    ld = Q.shape[1]
    a = og.batch_view(og.widen(Q), g, H, s_len * ld, d, s_len, d)
    b = og.batch_view(og.widen(K), g, H, s_len * ld, d, s_len, d)
    return np.ascontiguousarray(a), np.ascontiguousarray(b.T)


def run_scores(Q, K, n_seq, H, s_len, d, tile, S, out_dtype=torch.float32, task_ids=None):
    G = n_seq * H
    plan = cleave.plan_batched(s_len, s_len, d, tile, tile, S, G)
    ld = Q.shape[1]
    dQ, dK = Q.cuda(), K.cuda()
    parts = torch.full((plan.partial_elems,), float("nan"), dtype=torch.float32, device="cuda")
    C = torch.full((G * s_len, s_len), float("nan"), dtype=out_dtype, device="cuda")
    cleave.execute_batched(plan, dQ, (s_len * ld, d), dK, (s_len * ld, d), H, parts, 0, 1, task_ids=task_ids)
    cleave.reduce_batched(plan, parts, C, (H * s_len * s_len, s_len * s_len), H)
    torch.cuda.synchronize()
    return plan, parts, C


@pytest.mark.parametrize("dtype,n_seq,H,s_len,d,tile,S", [
    ("bf16", 2, 3, 192, 64, 128, 1),      # ragged tiles, direct path
    ("bf16", 1, 4, 320, 128, 256, 2),     # large class, two chunks of 64
    ("bf16", 2, 2, 100, 24, 64, 1),       # nothing a multiple of 8 in s: guarded path
    ("f32", 2, 2, 96, 40, 64, 2),
])
def test_batched_scores_match_oracle(dtype, n_seq, H, s_len, d, tile, S):
    Q = make_matrix(81, n_seq * s_len, H * d, dtype)
    K = make_matrix(82, n_seq * s_len, H * d, dtype)
    plan, parts, C = run_scores(Q, K, n_seq, H, s_len, d, tile, S)
    tasks, elems = planner.plan_batched(s_len, s_len, d, tile, tile, S, n_seq * H)
    assert plan.tasks.tobytes() == tasks.tobytes()
    ph, Ch = parts.cpu().numpy(), C.cpu().numpy()
    assert not np.isnan(ph).any() and not np.isnan(Ch).any()
    for g in range(n_seq * H):
        opA, opB = member_operands(Q, K, g, H, s_len, d)
        ref = og.gemm(opA, opB)
        got = Ch[g * s_len:(g + 1) * s_len]
        assert og.rel_frobenius(got, ref) <= TOL[dtype], g
        mine = tasks[tasks["gemm_id"] == g]
        for t in mine:
            blk = og.task_block(opA, opB, t)
            off = int(t["partial_off"])
            gotb = ph[off:off + blk.size].reshape(blk.shape)
            assert np.linalg.norm(gotb - blk) <= TOL[dtype] * (np.linalg.norm(blk) + np.linalg.norm(ref) / np.sqrt(ref.size))
        # aggregation of this member, bitwise the oracle's fp32 fold of the same partials
        local = mine.copy()
        base = int(local["partial_off"][0])
        local["partial_off"] -= base
        fold = og.reduce_partials(local, ph[base:base + S * s_len * s_len], s_len, s_len)
        assert np.array_equal(fold, got)


def test_batched_scores_integer_inputs_are_exact():
    n_seq, H, s_len, d = 2, 2, 256, 128
    Q = make_matrix(83, n_seq * s_len, H * d, "bf16", integer_valued=True)
    K = make_matrix(84, n_seq * s_len, H * d, "bf16", integer_valued=True)
    _, _, C = run_scores(Q, K, n_seq, H, s_len, d, 128, 2)
    Ch = C.cpu().numpy()
    for g in range(n_seq * H):
        opA, opB = member_operands(Q, K, g, H, s_len, d)
        assert np.array_equal(Ch[g * s_len:(g + 1) * s_len], og.gemm(opA, opB))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_batched_pv_layout_with_strided_output(dtype):
    """O_g = P_g V_g: P contiguous per member (s x s), V token-major [tokens, H*d] read as
    K x N, result written into token-major O."""
    n_seq, H, s_len, d, S = 2, 3, 256, 64, 2
    G = n_seq * H
    P = make_matrix(85, G * s_len, s_len, dtype)
    V = make_matrix(86, n_seq * s_len, H * d, dtype, std=0.02)
    ldv = H * d
    plan = cleave.plan_batched(s_len, d, s_len, 128, 64, S, G)
    parts = torch.empty(plan.partial_elems, dtype=torch.float32, device="cuda")
    O = torch.full((n_seq * s_len, H * d), float("nan"), dtype=torch.float32, device="cuda")
    cleave.execute_batched(plan, P.cuda(), (H * s_len * s_len, s_len * s_len), V.cuda(), (s_len * ldv, d), H, parts, 0, 0)
    cleave.reduce_batched(plan, parts, O, (s_len * ldv, d), H)
    torch.cuda.synchronize()
    Oh = O.cpu().numpy()
    assert not np.isnan(Oh).any()
    Pw, Vw = og.widen(P), og.widen(V)
    for g in range(G):
        o, i = divmod(g, H)
        opA = np.ascontiguousarray(og.batch_view(Pw, g, H, H * s_len * s_len, s_len * s_len, s_len, s_len))
        opB = np.ascontiguousarray(og.batch_view(Vw, g, H, s_len * ldv, d, s_len, d))
        ref = og.gemm(opA, opB)
        got = Oh[o * s_len:(o + 1) * s_len, i * d:(i + 1) * d]
        assert og.rel_frobenius(got, ref) <= TOL[dtype], g


def test_batched_reissue_is_bitwise_and_touches_only_its_blocks():
    n_seq, H, s_len, d = 2, 4, 256, 128
    Q = make_matrix(87, n_seq * s_len, H * d, "bf16")
    K = make_matrix(88, n_seq * s_len, H * d, "bf16")
    plan, parts, _ = run_scores(Q, K, n_seq, H, s_len, d, 128, 1)
    first = parts.clone()
    tasks = plan.tasks
    lost = [1, 7, 12, len(tasks) - 1, 18]
    for i in lost:
        off = int(tasks[i]["partial_off"])
        parts[off:off + int(tasks[i]["m_len"]) * int(tasks[i]["n_len"])] = float("nan")
    ld = Q.shape[1]
    cleave.execute_batched(plan, Q.cuda(), (s_len * ld, d), K.cuda(), (s_len * ld, d), H, parts, 0, 1, task_ids=lost)
    torch.cuda.synchronize()
    assert torch.equal(parts.view(torch.int32), first.view(torch.int32))


def test_attention_scores_at_llama7b_layer_size_sampled():
    """128 score GEMMs of 1024 x 128 x 1024 (4 sequences x 32 heads): every member by
    the projection identity, sampled members in full."""
    n_seq, H, s_len, d = 4, 32, 1024, 128
    Q = make_matrix(91, n_seq * s_len, H * d, "bf16")
    K = make_matrix(92, n_seq * s_len, H * d, "bf16")
    plan, parts, C = run_scores(Q, K, n_seq, H, s_len, d, 512, 1)
    assert plan.num_tasks == 128 * 4
    Ch = C.cpu().numpy()
    rng = np.random.default_rng(93)
    full = {0, n_seq * H - 1} | {int(g) for g in rng.integers(0, n_seq * H, 3)}
    for g in range(n_seq * H):
        opA, opB = member_operands(Q, K, g, H, s_len, d)
        got = Ch[g * s_len:(g + 1) * s_len]
        assert og.projection_check(opA, opB, got, seed=1000 + g) < 1e-4, g
        if g in full:
            assert og.rel_frobenius(got, og.gemm(opA, opB)) <= TOL["bf16"], g
    print("scores kernel", plan.last_kernel)


def test_batched_and_plain_calls_do_not_mix():
    bp = cleave.plan_batched(64, 64, 64, 32, 32, 1, 4)
    pp = cleave.plan_uniform(64, 64, 64, 32, 32, 1)
    A = torch.zeros(256, 64, dtype=torch.bfloat16, device="cuda")
    one = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda")
    parts = torch.zeros(bp.partial_elems, device="cuda")
    C = torch.zeros(256, 64, device="cuda")
    with pytest.raises(cleave.CleaveError):
        cleave.execute_batched(pp, A, (0, 0), A, (0, 0), 1, parts)
    with pytest.raises(cleave.CleaveError):
        cleave.execute(bp, one, one, parts)
    with pytest.raises(cleave.CleaveError):
        cleave.execute_batched(bp, A, (0, 64 * 64), A, (0, 64 * 64), 3, parts)     # 3 does not divide 4
    with pytest.raises(cleave.CleaveError):
        cleave.reduce(bp, parts, C[:64])
    with pytest.raises(cleave.CleaveError):
        cleave.execute_batched(bp, A, (-1, 0), A, (0, 0), 4, parts)
