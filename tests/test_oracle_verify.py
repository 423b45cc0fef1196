"""Pins for the oracle of the returned-block check (Sec. 6 "Robustness to
poisoning attacks"): brute force with Python integers on tiny shapes, the exact
identity r^T (A B) s = (A^T r)^T (B s) on integer-valued inputs, the exact size
of the residual a single corrupted entry leaves, the chunk restriction of the
K-split extension, additivity over a tile's splits, and the bound
|rhs| <= scale."""
import numpy as np
import pytest

from oracle import gemm as og
from oracle import planner
from oracle import verify as ov
from workloads.tensors import make_matrix, make_probe_vectors


def n_partial(tasks):
    return int(sum(int(t["m_len"]) * int(t["n_len"]) for t in tasks))


def int_inputs(seed, M, N, K):
    rng = np.random.default_rng(seed)
    a = rng.integers(-5, 6, (M, K))
    b = rng.integers(-5, 6, (K, N))
    r = rng.integers(-3, 4, M)
    s = rng.integers(-3, 4, N)
    return a, b, r, s


def brute(a, b, P, r, s, t):
    """lhs, rhs, scale by plain loops over Python integers."""
    m0, ml, n0, nl, k0, kl = (int(t[f]) for f in ("m0", "m_len", "n0", "n_len", "k0", "k_len"))
    lhs = sum(int(r[m0 + i]) * int(P[i][j]) * int(s[n0 + j]) for i in range(ml) for j in range(nl))
    rhs = 0
    scale = 0
    for k in range(k0, k0 + kl):
        u = sum(int(a[m0 + i][k]) * int(r[m0 + i]) for i in range(ml))
        v = sum(int(b[k][n0 + j]) * int(s[n0 + j]) for j in range(nl))
        ua = sum(abs(int(a[m0 + i][k])) * abs(int(r[m0 + i])) for i in range(ml))
        va = sum(abs(int(b[k][n0 + j])) * abs(int(s[n0 + j])) for j in range(nl))
        rhs += u * v
        scale += ua * va
    return lhs, rhs, scale


@pytest.mark.parametrize("M,N,K,tm,tn,S", [(5, 7, 6, 2, 3, 2), (8, 4, 9, 8, 4, 3), (3, 3, 4, 1, 2, 1)])
def test_brute_force_on_tiny_shapes(M, N, K, tm, tn, S):
    a, b, r, s = int_inputs(10 * M + N, M, N, K)
    tasks, _ = planner.plan_uniform(M, N, K, tm, tn, S)
    opA, opB = a.astype(np.float64), b.astype(np.float64)
    rng = np.random.default_rng(3)
    for t in tasks:
        # an arbitrary integer block, not the product: lhs and rhs are independent sums
        P = rng.integers(-20, 21, (int(t["m_len"]), int(t["n_len"])))
        lhs, rhs, scale, _ = ov.verify_task(opA, opB, P, t, r, s, 0.0)
        assert (lhs, rhs, scale) == tuple(float(x) for x in brute(a, b, P.tolist(), r, s, t))


def test_identity_is_exact_for_the_true_blocks_and_accepts_at_zero_tolerance():
    M, N, K = 24, 20, 32
    a, b, r, s = int_inputs(7, M, N, K)
    tasks, _ = planner.plan_uniform(M, N, K, 8, 8, 4)      # non-square blocks of a non-square product
    opA, opB = a.astype(np.float64), b.astype(np.float64)
    partials = og.execute_tasks(tasks, opA, opB, n_partial(tasks))
    lhs, rhs, scale, accept = ov.verify_tasks(tasks, opA, opB, partials, r, s, 0.0)
    assert np.array_equal(lhs, rhs)
    assert accept.all()
    assert np.all(scale >= np.abs(rhs))


def test_single_corrupted_entry_leaves_exactly_its_weighted_size():
    M, N, K = 16, 12, 8
    a, b, _, _ = int_inputs(11, M, N, K)
    r, s = (v.numpy() for v in make_probe_vectors(5, M, N, kind="sign"))
    tasks, _ = planner.plan_uniform(M, N, K, 8, 6, 2)
    opA, opB = a.astype(np.float64), b.astype(np.float64)
    t = tasks[3]
    P = og.task_block(opA, opB, t)
    P[5, 2] += 3.0
    lhs, rhs, scale, accept = ov.verify_task(opA, opB, P, t, r, s, 0.0)
    assert abs(lhs - rhs) == 3.0 and not accept
    # the threshold sits where the rule says: |lhs - rhs| <= tol * scale
    assert ov.verify_task(opA, opB, P, t, r, s, 3.0 / scale * (1 + 1e-12))[3]
    assert not ov.verify_task(opA, opB, P, t, r, s, 3.0 / scale * (1 - 1e-12))[3]


def test_block_of_another_chunk_or_tile_is_rejected():
    M, N, K = 16, 16, 16
    a, b, r, s = int_inputs(13, M, N, K)
    r = np.where(r == 0, 1, r)
    s = np.where(s == 0, 1, s)
    tasks, _ = planner.plan_uniform(M, N, K, 8, 8, 2)
    opA, opB = a.astype(np.float64), b.astype(np.float64)
    blocks = [og.task_block(opA, opB, t) for t in tasks]
    wrong = 0
    for i, t in enumerate(tasks):
        for j in range(len(tasks)):
            ok = ov.verify_task(opA, opB, blocks[j], t, r, s, 0.0)[3]
            assert ok or i != j
            wrong += (ok and i != j)
    assert wrong == 0     # with these seeds no foreign block passes by accident


def test_lhs_is_additive_over_the_splits_of_a_tile():
    M, N, K = 12, 10, 24
    a, b, r, s = int_inputs(17, M, N, K)
    tasks, _ = planner.plan_uniform(M, N, K, 12, 10, 3)
    opA, opB = a.astype(np.float64), b.astype(np.float64)
    partials = og.execute_tasks(tasks, opA, opB, n_partial(tasks))
    lhs, rhs, _, _ = ov.verify_tasks(tasks, opA, opB, partials, r, s, 0.0)
    full = float(r @ (opA @ opB) @ s)
    assert lhs.sum() == full and rhs.sum() == full


def test_scale_equals_rhs_for_nonnegative_inputs_and_bounds_it_otherwise():
    rng = np.random.default_rng(19)
    opA = rng.random((9, 7))
    opB = rng.random((7, 5))
    r, s = rng.random(9), rng.random(5)
    t = planner.plan_uniform(9, 5, 7, 9, 5, 1)[0][0]
    lhs, rhs, scale, accept = ov.verify_task(opA, opB, opA @ opB, t, r, s, 1e-14)
    assert abs(scale - rhs) <= 1e-13 * scale and accept
    lhs, rhs, scale, _ = ov.verify_task(-opA, opB, -(opA @ opB), t, r, s, 1e-14)
    assert rhs < 0 and abs(scale + rhs) <= 1e-13 * scale


def test_rounded_fp32_blocks_of_bf16_inputs_pass_a_loose_tolerance_only():
    # fp32 blocks of bf16 inputs differ from the exact product by rounding: the residual is
    # far below 1e-6 * scale and far above 0.
    M, N, K = 64, 48, 256
    A = make_matrix(21, M, K)
    B = make_matrix(22, K, N, std=0.02)
    r, s = (v.numpy() for v in make_probe_vectors(23, M, N))
    opA, opB = og.logical_operands(A, 0, B, 0)
    tasks, _ = planner.plan_uniform(M, N, K, 32, 48, 2)
    for t in tasks:
        P32 = og.task_block(opA, opB, t).astype(np.float32)
        lhs, rhs, scale, ok = ov.verify_task(opA, opB, P32, t, r, s, 1e-6)
        assert ok and 0 < abs(lhs - rhs) < 1e-7 * scale
        assert not ov.verify_task(opA, opB, P32, t, r, s, 0.0)[3]
