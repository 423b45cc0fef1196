"""Pins for the oracle's arithmetic: exact brute force on tiny shapes (integer
arithmetic in Python), textbook special cases, a library fp64 matmul, exact
integer-valued inputs, the decomposition invariants the paper fixes (sum of
task outputs == undecomposed GEMM, independence of the tiling) and the fixed
fold order of the aggregator."""
import numpy as np
import pytest
import torch

from oracle import gemm as og
from oracle import planner
from workloads.tensors import make_matrix


def python_matmul(a, b):
    """Exact integer matmul on nested lists, plain loops."""
    M, K, N = len(a), len(b), len(b[0])
    return [[sum(a[i][k] * b[k][j] for k in range(K)) for j in range(N)] for i in range(M)]


def stored(logical, trans):
    """Stored layout of a logical operand under the boundary's convention."""
    return np.ascontiguousarray(logical.T) if trans else np.ascontiguousarray(logical)


@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (2, 3, 4), (5, 2, 7), (8, 7, 3)])
def test_gemm_brute_force_all_layouts(M, N, K, transA, transB):
    rng = np.random.default_rng(100 * M + 10 * N + K)
    a = rng.integers(-9, 10, (M, K))
    b = rng.integers(-9, 10, (K, N))
    expect = np.array(python_matmul(a.tolist(), b.tolist()), dtype=np.float64)
    opA, opB = og.logical_operands(stored(a.astype(np.float32), transA), transA,
                                   stored(b.astype(np.float32), transB), transB)
    assert opA.shape == (M, K) and opB.shape == (K, N)
    assert np.array_equal(og.gemm(opA, opB), expect)


def test_gemm_identity_and_column_sums():
    rng = np.random.default_rng(5)
    a = rng.standard_normal((37, 29))
    assert np.array_equal(og.gemm(a, np.eye(29)), a)                 # B = I  =>  C = A exactly
    ones = np.ones((3, 37))
    got = og.gemm(ones, a)                                           # rows of ones => column sums
    col = np.zeros(29)
    for i in range(37):                                              # same ascending order
        col = col + a[i]
    assert np.array_equal(got, np.tile(col, (3, 1)))


def test_gemm_matches_library_fp64():
    rng = np.random.default_rng(11)
    a = rng.standard_normal((150, 170))
    b = rng.standard_normal((170, 130))
    ref = a @ b
    assert og.rel_frobenius(og.gemm(a, b), ref) < 1e-14
    # a sub-range of the inner dimension, through strided row/column views
    big = rng.standard_normal((200, 300))
    rows = big[20:90, :170]
    assert not rows.flags["C_CONTIGUOUS"]
    ref = rows[:, 40:120] @ b[40:120]
    assert og.rel_frobenius(og.gemm(rows, b, 40, 120), ref) < 1e-14


def test_bf16_and_fp32_inputs_are_widened_exactly():
    x = make_matrix(3, 16, 24, "bf16")
    w = og.widen(x)
    assert w.dtype == np.float64
    assert torch.equal(torch.from_numpy(w).to(torch.bfloat16), x)    # round trip is lossless
    bits = x.view(torch.int16).numpy().astype(np.uint16).astype(np.uint32) << 16
    assert np.array_equal(bits.view(np.float32).astype(np.float64), w)  # bf16 = top half of fp32
    y = make_matrix(4, 8, 8, "f32")
    assert np.array_equal(og.widen(y), y.numpy().astype(np.float64))


@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0)])
def test_integer_inputs_are_exact_for_any_decomposition(transA, transB):
    M, N, K = 96, 80, 160
    a = make_matrix(21, M, K, "bf16", integer_valued=True)
    b = make_matrix(22, K, N, "bf16", integer_valued=True)
    exact = (a.to(torch.int64) @ b.to(torch.int64)).numpy().astype(np.float64)
    A = a.t().contiguous() if transA else a
    B = b.t().contiguous() if transB else b
    opA, opB = og.logical_operands(A, transA, B, transB)
    assert np.array_equal(og.gemm(opA, opB), exact)
    for tm, tn, S in [(32, 32, 1), (40, 48, 4), (96, 80, 5), (17, 23, 8)]:
        tasks, elems = planner.plan_uniform(M, N, K, tm, tn, S)
        parts = og.execute_tasks(tasks, opA, opB, elems)
        assert np.array_equal(og.reduce_partials(tasks, parts, M, N), exact)
        p32 = parts.astype(np.float32)
        assert np.array_equal(og.reduce_partials(tasks, p32, M, N).astype(np.float64), exact)


def test_sum_of_task_outputs_equals_undecomposed_gemm():
    M, N, K = 130, 150, 190
    a = og.widen(make_matrix(31, M, K, "bf16"))
    b = og.widen(make_matrix(32, K, N, "bf16", std=0.02))
    full = og.gemm(a, b)
    assert og.rel_frobenius(full, a @ b) < 1e-14
    results = []
    for tm, tn, S in [(130, 150, 1), (64, 64, 2), (50, 70, 4), (128, 32, 8)]:
        tasks, elems = planner.plan_uniform(M, N, K, tm, tn, S)
        parts = og.execute_tasks(tasks, a, b, elems)
        C = og.reduce_partials(tasks, parts, M, N)
        assert og.rel_frobenius(C, full) < 1e-13
        results.append(C)
    assert np.array_equal(results[0], full)        # S = 1: assembling blocks changes nothing
    # heterogeneous tiling of the same GEMM
    tasks, elems = planner.plan_explicit(M, N, K, [100, 30], [[150], [64, 86]], [2, 1, 4])
    C = og.reduce_partials(tasks, og.execute_tasks(tasks, a, b, elems), M, N)
    assert og.rel_frobenius(C, full) < 1e-13


def test_task_block_is_rows_of_A_times_columns_of_B():
    a = og.widen(make_matrix(41, 40, 64, "f32"))
    b = og.widen(make_matrix(42, 64, 56, "f32"))
    tasks, _ = planner.plan_uniform(40, 56, 64, 16, 24, 2)
    t = tasks[7]   # tile 3 (row 1, col 0), split 1
    assert (int(t["m0"]), int(t["n0"]), int(t["k0"]), int(t["k_len"])) == (16, 0, 32, 32)
    ref = a[16:32, 32:64] @ b[32:64, 0:24]
    assert og.rel_frobenius(og.task_block(a, b, t), ref) < 1e-14
    blk = og.output_block(a, b, 8, 9, 30, 11)
    assert og.rel_frobenius(blk, (a @ b)[8:17, 30:41]) < 1e-14


def test_reissued_tasks_overwrite_only_their_blocks():
    a = og.widen(make_matrix(51, 48, 32, "f32"))
    b = og.widen(make_matrix(52, 32, 40, "f32"))
    tasks, elems = planner.plan_uniform(48, 40, 32, 16, 16, 2)
    parts = og.execute_tasks(tasks, a, b, elems)
    poisoned = parts.copy()
    lost = [3, 11, 4]
    for i in lost:
        off = int(tasks[i]["partial_off"])
        poisoned[off:off + int(tasks[i]["m_len"]) * int(tasks[i]["n_len"])] = np.nan
    assert np.isnan(poisoned).sum() == 256 + 128 + 128
    og.execute_tasks(tasks, a, b, elems, out=poisoned, task_ids=lost)
    assert np.array_equal(poisoned, parts)


def test_fold_order_is_left_to_right_in_fp32():
    # (1e8 + -1e8) + 1 = 1, but 1e8 + (-1e8 + 1) = 0 in fp32.
    tasks, elems = planner.plan_uniform(1, 1, 3, 1, 1, 3)
    parts = np.array([1e8, -1e8, 1.0], dtype=np.float32)
    assert og.reduce_partials(tasks, parts, 1, 1)[0, 0] == np.float32(1.0)
    parts = np.array([1.0, 1e8, -1e8], dtype=np.float32)
    assert og.reduce_partials(tasks, parts, 1, 1)[0, 0] == np.float32(0.0)
    # S = 1 is a bitwise copy; S = 2 is one IEEE single add per element.
    rng = np.random.default_rng(9)
    p = rng.standard_normal(2 * 24 * 20).astype(np.float32)
    t1, _ = planner.plan_uniform(24, 40, 4, 24, 20, 1)
    assert np.array_equal(og.reduce_partials(t1, p, 24, 40)[:, :20].reshape(-1), p[:480])
    t2, _ = planner.plan_uniform(24, 20, 4, 24, 20, 2)
    assert np.array_equal(og.reduce_partials(t2, p, 24, 20).reshape(-1), p[:480] + p[480:])
    # S = 4 against an explicit numpy fp32 left fold
    t4, _ = planner.plan_uniform(8, 8, 8, 8, 8, 4)
    q = (rng.standard_normal(256) * 1e4).astype(np.float32)
    expect = ((q[:64] + q[64:128]) + q[128:192]) + q[192:]
    assert np.array_equal(og.reduce_partials(t4, q, 8, 8).reshape(-1), expect)


def test_projection_check_accepts_product_and_detects_one_bad_entry():
    rng = np.random.default_rng(13)
    a = rng.standard_normal((90, 70))
    b = rng.standard_normal((70, 110))
    c = og.gemm(a, b)
    assert og.projection_check(a, b, c, seed=1) < 1e-13
    bad = c.copy()
    bad[17, 60] += 1.0
    assert og.projection_check(a, b, bad, seed=1) > 1e-6
    assert og.projection_check(a, b, c.T.copy().T * (1 + 1e-3), seed=2) > 1e-5


def test_batch_view_is_the_head_slice_of_a_token_major_activation():
    # Q stored [T, H*d], token-major: sequence o, head i is rows o*s..(o+1)*s, columns i*d..(i+1)*d
    s_len, H, d, n_seq = 6, 3, 4, 2
    Q = np.arange(n_seq * s_len * H * d, dtype=np.float64).reshape(n_seq * s_len, H * d)
    ld = H * d
    for g in range(n_seq * H):
        o, i = divmod(g, H)
        v = og.batch_view(Q, g, H, s_len * ld, d, s_len, d)
        assert np.array_equal(v, Q[o * s_len:(o + 1) * s_len, i * d:(i + 1) * d])
    # contiguous per-GEMM blocks (scores [n_seq*H, s, s]): stride s*s, ld = s
    P = np.arange(n_seq * H * s_len * s_len, dtype=np.float64).reshape(n_seq * H * s_len, s_len)
    for g in range(n_seq * H):
        v = og.batch_view(P, g, H, H * s_len * s_len, s_len * s_len, s_len, s_len)
        assert np.array_equal(v, P[g * s_len:(g + 1) * s_len, :])
    with pytest.raises(ValueError):
        og.batch_view(Q, n_seq * H, H, s_len * ld, d, s_len, d)


def test_rel_frobenius_hand_values():
    # the yard-stick of every parity bar: ||C - C_ref||_F / ||C_ref||_F
    ref = np.array([[3.0, 4.0]])                          # norm 5
    assert og.rel_frobenius(np.array([[3.0, 4.05]]), ref) == pytest.approx(0.01, rel=1e-12)
    ref = np.array([[1.0, 2.0], [2.0, 4.0]])              # norm sqrt(25) = 5
    got = ref + np.array([[0.3, 0.0], [0.0, -0.4]])       # difference norm 0.5
    assert og.rel_frobenius(got, ref) == pytest.approx(0.1, rel=1e-12)
    # not symmetric in its arguments (the reference normalises), exact zero for equal inputs,
    # absolute norm when the reference vanishes
    assert og.rel_frobenius(ref, got) != pytest.approx(0.1, rel=1e-6)
    assert og.rel_frobenius(ref, ref) == 0.0
    assert og.rel_frobenius(np.array([[0.6, 0.8]]), np.zeros((1, 2))) == pytest.approx(1.0, rel=1e-12)
    # fp32 input is widened, not rounded further
    assert og.rel_frobenius(np.array([[3.0, 4.5]], dtype=np.float32), np.array([[3.0, 4.0]])) == pytest.approx(0.1, rel=1e-12)
