"""GPU parity of the returned-block check (cleave_verify through the C ABI)
against its fp64 oracle.

The partial blocks handed to both sides are synthetic: the oracle's own fp64
blocks rounded to fp32 (some of them corrupted on purpose -- a mistake planted
in the data, on the CPU), or seeded random values.  Bars: lhs, rhs, scale within
1e-12 of the size of the sums they accumulate (both sides sum in fp64, in
different orders); accept flags identical (the cases sit far from the
threshold); everything bit-exact for integer-valued inputs.
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

pytestmark = pytest.mark.gpu

LAYOUTS = [(0, 0), (0, 1), (1, 0), (1, 1)]


def gpu_verify(plan, A, B, transA, transB, partials, r, s, tol):
    n = plan.num_tasks
    out = {k: torch.full((n,), float("nan"), dtype=torch.float64, device="cuda") for k in ("lhs", "rhs", "scale")}
    accept = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    cleave.verify(plan, A.cuda(), B.cuda(), torch.from_numpy(partials).cuda(), r.cuda(), s.cuda(), tol,
                  accept, out["lhs"], out["rhs"], out["scale"], transA=transA, transB=transB)
    torch.cuda.synchronize()
    return out["lhs"].cpu().numpy(), out["rhs"].cpu().numpy(), out["scale"].cpu().numpy(), accept.cpu().numpy()


def oracle_partials(tasks, opA, opB, elems, corrupt=()):
    """fp32 roundings of the oracle's blocks; tasks listed in `corrupt` get one entry changed."""
    parts = og.execute_tasks(tasks, opA, opB, elems).astype(np.float32)
    for i in corrupt:
        t = tasks[i]
        cnt = int(t["m_len"]) * int(t["n_len"])
        pos = int(t["partial_off"]) + (7 * i + 3) % cnt
        parts[pos] += np.float32(1000.0)   # large against tol * scale / |r_i s_j| for these shapes
    return parts


def lhs_size(tasks, parts, r, s):
    """sum |r_i| |P_ij| |s_j| per task: the size of what lhs accumulates."""
    out = np.zeros(len(tasks))
    for i, t in enumerate(tasks):
        m0, ml, n0, nl = (int(t[f]) for f in ("m0", "m_len", "n0", "n_len"))
        off = int(t["partial_off"])
        P = np.abs(parts[off:off + ml * nl].astype(np.float64)).reshape(ml, nl)
        out[i] = np.abs(r[m0:m0 + ml]) @ P @ np.abs(s[n0:n0 + nl])
    return out


def compare(tasks, got, ref, sizes):
    lhs, rhs, scale, accept = got
    lhs_r, rhs_r, scale_r, accept_r = ref
    assert np.all(np.abs(lhs - lhs_r) <= 1e-12 * sizes + 1e-300)
    assert np.all(np.abs(rhs - rhs_r) <= 1e-12 * scale_r + 1e-300)
    assert np.all(np.abs(scale - scale_r) <= 1e-12 * scale_r + 1e-300)
    assert np.array_equal(accept, accept_r)


# several tiles and a ragged tail; the first shapes keep the 16-byte paths, the others do not
SHAPES = [
    (256, 384, 192, 128, 128, 3), (640, 392, 512, 256, 256, 2), (300, 200, 72, 128, 128, 3),
    (37, 29, 50, 16, 8, 2), (130, 150, 10, 64, 64, 3), (96, 260, 64, 96, 260, 1),
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("transA,transB", LAYOUTS)
@pytest.mark.parametrize("M,N,K,tm,tn,S", SHAPES)
def test_verify_matches_oracle(M, N, K, tm, tn, S, transA, transB, dtype):
    A_log = make_matrix(31 + M, M, K, dtype)
    B_log = make_matrix(32 + N, K, N, dtype, std=0.02)
    A, B = stored(A_log, transA), stored(B_log, transB)
    r, s = make_probe_vectors(33 + K, M, N)
    plan = cleave.plan_uniform(M, N, K, tm, tn, S)
    tasks, elems = planner.plan_uniform(M, N, K, tm, tn, S)
    opA, opB = og.logical_operands(A, transA, B, transB)
    bad = list(range(1, len(tasks), 3))
    parts = oracle_partials(tasks, opA, opB, elems, corrupt=bad)
    tol = 1e-6
    ref = ov.verify_tasks(tasks, opA, opB, parts, r.numpy(), s.numpy(), tol)
    got = gpu_verify(plan, A, B, transA, transB, parts, r, s, tol)
    compare(tasks, got, ref, lhs_size(tasks, parts, r.numpy(), s.numpy()))
    # the planted corruptions, and only they, are rejected
    assert set(np.flatnonzero(got[3] == 0)) == set(bad)


@pytest.mark.parametrize("transA,transB", LAYOUTS)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_verify_is_exact_on_integer_inputs(transA, transB, dtype):
    M, N, K, tm, tn, S = 384, 264, 256, 128, 88, 4
    A_log = make_matrix(41, M, K, dtype, integer_valued=True)
    B_log = make_matrix(42, K, N, dtype, integer_valued=True)
    A, B = stored(A_log, transA), stored(B_log, transB)
    r, s = make_probe_vectors(43, M, N, kind="sign")
    plan = cleave.plan_uniform(M, N, K, tm, tn, S)
    tasks, elems = planner.plan_uniform(M, N, K, tm, tn, S)
    opA, opB = og.logical_operands(A, transA, B, transB)
    parts = og.execute_tasks(tasks, opA, opB, elems).astype(np.float32)   # exact integers
    bad = [0, 5, len(tasks) - 1]
    for i in bad:
        parts[int(tasks[i]["partial_off"]) + 11 * i] += 1.0
    ref = ov.verify_tasks(tasks, opA, opB, parts, r.numpy(), s.numpy(), 0.0)
    lhs, rhs, scale, accept = gpu_verify(plan, A, B, transA, transB, parts, r, s, 0.0)
    assert np.array_equal(lhs, ref[0]) and np.array_equal(rhs, ref[1]) and np.array_equal(scale, ref[2])
    assert np.array_equal(accept, ref[3])
    assert np.array_equal(np.abs(lhs - rhs) == 1.0, accept == 0)
    assert set(np.flatnonzero(accept == 0)) == set(bad)


def test_verify_heterogeneous_tiling():
    M, N, K = 1536, 1280, 512
    band_h, col_w, ks = draw_explicit_tiling(M, N, K, seed=77)
    plan = cleave.plan_explicit(M, N, K, band_h, col_w, ks)
    tasks, elems = planner.plan_explicit(M, N, K, band_h, col_w, ks)
    assert plan.tasks.tobytes() == tasks.tobytes()
    A = make_matrix(51, M, K)
    B = make_matrix(52, K, N, std=0.02)
    r, s = make_probe_vectors(53, M, N)
    opA, opB = og.logical_operands(A, 0, B, 0)
    bad = list(range(0, len(tasks), 7))
    parts = oracle_partials(tasks, opA, opB, elems, corrupt=bad)
    ref = ov.verify_tasks(tasks, opA, opB, parts, r.numpy(), s.numpy(), 1e-6)
    got = gpu_verify(plan, A, B, 0, 0, parts, r, s, 1e-6)
    compare(tasks, got, ref, lhs_size(tasks, parts, r.numpy(), s.numpy()))
    assert set(np.flatnonzero(got[3] == 0)) == set(bad)


def test_verify_after_execute_accepts_honest_blocks_and_flags_tampered_ones():
    """End to end on the device: blocks written by cleave_execute pass, blocks
    overwritten afterwards do not (a property; no oracle values involved)."""
    M, N, K, transA, transB = 1024, 1536, 2048, 0, 0
    A = make_matrix(61, M, K).cuda()
    B = make_matrix(62, K, N, std=0.02).cuda()
    r, s = (v.cuda() for v in make_probe_vectors(63, M, N))
    plan = cleave.plan_uniform(M, N, K, 512, 512, 4)
    parts = torch.empty(plan.partial_elems, dtype=torch.float32, device="cuda")
    cleave.execute(plan, A, B, parts, transA, transB)
    accept = torch.empty(plan.num_tasks, dtype=torch.int32, device="cuda")
    cleave.verify(plan, A, B, parts, r, s, 1e-6, accept)
    assert bool((accept == 1).all())
    tasks = plan.tasks
    bad = [2, 9, 17]
    for i in bad:
        parts[int(tasks[i]["partial_off"]) + 1000 + i] += 1000.0
    cleave.verify(plan, A, B, parts, r, s, 1e-6, accept)
    torch.cuda.synchronize()
    assert set(np.flatnonzero(accept.cpu().numpy() == 0)) == set(bad)


def test_verify_rejects_bad_arguments():
    plan = cleave.plan_uniform(64, 64, 64, 32, 32, 1)
    A = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda")
    parts = torch.zeros(plan.partial_elems, device="cuda")
    r = torch.zeros(64, device="cuda")
    accept = torch.zeros(plan.num_tasks, dtype=torch.int32, device="cuda")
    with pytest.raises(cleave.CleaveError) as e:
        cleave.verify(plan, A, A, parts, r, r, -1.0, accept)
    assert e.value.status == -1
    with pytest.raises(cleave.CleaveError):
        cleave.verify(plan, A, A, parts, r, r, float("nan"), accept)
    with pytest.raises(ValueError):
        cleave.verify(plan, A, A, parts, r[:10], r, 0.0, accept)


def _full_size_check(g, plan, tasks, cfg, cache, seed, n_samples=6):
    """cleave_verify over a whole GEMM of a benchmark configuration; seeded random
    fp32 values stand in for the partial blocks; sampled tasks (always the last,
    ragged one) against the oracle, one by one."""
    from workloads import make_gemm_operands
    A, B = make_gemm_operands(cfg, g, cache=cache)
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    parts = torch.randn(plan.partial_elems, generator=gen, dtype=torch.float32)
    r, s = make_probe_vectors(seed + 1, g.M, g.N)
    n = plan.num_tasks
    lhs, rhs, scale = (torch.empty(n, dtype=torch.float64, device="cuda") for _ in range(3))
    accept = torch.empty(n, dtype=torch.int32, device="cuda")
    cleave.verify(plan, A.cuda(), B.cuda(), parts.cuda(), r.cuda(), s.cuda(), 1e-6, accept, lhs, rhs, scale,
                  transA=g.transA, transB=g.transB)
    torch.cuda.synchronize()
    lhs, rhs, scale, accept = (x.cpu().numpy() for x in (lhs, rhs, scale, accept))
    opA, opB = og.logical_operands(A, g.transA, B, g.transB)
    rng = np.random.default_rng(seed)
    picks = sorted({n - 1, 0} | {int(i) for i in rng.integers(0, n, n_samples)})
    pn, rn, sn = parts.numpy(), r.numpy(), s.numpy()
    for i in picks:
        t = tasks[i]
        off, cnt = int(t["partial_off"]), int(t["m_len"]) * int(t["n_len"])
        l, h, sc, ok = ov.verify_task(opA, opB, pn[off:off + cnt], t, rn, sn, 1e-6)
        size = lhs_size(tasks[i:i + 1], pn, rn, sn)[0]
        assert abs(lhs[i] - l) <= 1e-12 * size, (g.name, i)
        assert abs(rhs[i] - h) <= 1e-12 * sc and abs(scale[i] - sc) <= 1e-12 * sc, (g.name, i)
        assert accept[i] == int(ok), (g.name, i)
    assert accept.sum() <= n // 20      # random blocks are not the products; a few may pass by chance


def test_verify_c3_full_size_sampled():
    from workloads import layer_config
    cfg = layer_config("c3")
    cache = {}
    for gid, g in enumerate(cfg.gemms):
        if g.name not in ("q.fwd", "gate.fwd", "down.dx", "up.dw"):
            continue
        plan = cleave.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit, gemm_id=gid)
        tasks, _ = planner.plan_uniform(g.M, g.N, g.K, cfg.tile_m, cfg.tile_n, cfg.ksplit, gemm_id=gid)
        _full_size_check(g, plan, tasks, cfg, cache, seed=7000 + gid)
        print("c3 verify", g.name, plan.num_tasks, "tasks", flush=True)


def test_verify_c4_heterogeneous_full_size_sampled():
    from workloads import layer_config
    from workloads.configs import C4_TILING_SEED
    cfg = layer_config("c4")
    cache = {}
    for gid, g in enumerate(cfg.gemms):
        if g.name not in ("gate.fwd", "down.dw"):
            continue
        band_h, col_w, ks = draw_explicit_tiling(g.M, g.N, g.K, C4_TILING_SEED + gid)
        plan = cleave.plan_explicit(g.M, g.N, g.K, band_h, col_w, ks, gemm_id=gid)
        tasks, _ = planner.plan_explicit(g.M, g.N, g.K, band_h, col_w, ks, gemm_id=gid)
        _full_size_check(g, plan, tasks, cfg, cache, seed=7100 + gid)
        print("c4 verify", g.name, plan.num_tasks, "tasks", flush=True)


# ---- batched and grouped plans (the attention products; the GEMMs of a DAG level) ----

def oracle_batched(tasks, member_operands, parts, r, s, tol, per_member):
    """Per task of a batched list: the oracle's check with the member's operands and
    probe vectors.  member_operands(g) -> (opA, opB)."""
    n = len(tasks)
    lhs, rhs, scale, accept = np.zeros(n), np.zeros(n), np.zeros(n), np.zeros(n, dtype=np.int32)
    cache = {}
    for i, t in enumerate(tasks):
        g = int(t["gemm_id"])
        if g not in cache:
            cache[g] = member_operands(g)
        opA, opB = cache[g]
        off, cnt = int(t["partial_off"]), int(t["m_len"]) * int(t["n_len"])
        lhs[i], rhs[i], scale[i], ok = ov.verify_task(opA, opB, parts[off:off + cnt], t, r[g], s[g], tol)
        accept[i] = int(ok)
    return lhs, rhs, scale, accept


@pytest.mark.parametrize("integer", [False, True])
def test_verify_batched_attention_scores_matches_oracle(integer):
    """Q K^T per sequence and head as one batched task list over token-major Q, K
    (zero-copy strided views); blocks written by the library's own executor, one of
    them corrupted afterwards."""
    n_seq, H, s_len, d, tile = 2, 3, 192, 64, 128
    G, ld = n_seq * H, H * d
    Q = make_matrix(61, n_seq * s_len, ld, "bf16", integer_valued=integer)
    Kt = make_matrix(62, n_seq * s_len, ld, "bf16", integer_valued=integer)
    plan = cleave.plan_batched(s_len, s_len, d, tile, tile, 1, G)
    tasks, elems = planner.plan_batched(s_len, s_len, d, tile, tile, 1, G)
    assert plan.tasks.tobytes() == tasks.tobytes()
    dQ, dK = Q.cuda(), Kt.cuda()
    parts = torch.empty(elems, dtype=torch.float32, device="cuda")
    strides = (s_len * ld, d)
    cleave.execute_batched(plan, dQ, strides, dK, strides, H, parts, 0, 1)
    bad = [2, len(tasks) - 3]
    for i in bad:
        parts[int(tasks[i]["partial_off"]) + 11] += 1000.0
    gen = torch.Generator(device="cpu")
    gen.manual_seed(63)
    if integer:
        r = (torch.randint(0, 2, (G, s_len), generator=gen, dtype=torch.int32).float() * 2 - 1)
        s = (torch.randint(0, 2, (G, s_len), generator=gen, dtype=torch.int32).float() * 2 - 1)
    else:
        r = torch.randn((G, s_len), generator=gen)
        s = torch.randn((G, s_len), generator=gen)
    n = plan.num_tasks
    out = {k: torch.full((n,), float("nan"), dtype=torch.float64, device="cuda") for k in ("lhs", "rhs", "scale")}
    accept = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    cleave.verify_batched(plan, dQ, strides, dK, strides, H, parts, r.cuda(), s.cuda(), 1e-6, accept,
                          out["lhs"], out["rhs"], out["scale"], transA=0, transB=1)
    torch.cuda.synchronize()
    Qd, Kd = og.widen(Q), og.widen(Kt)

    def member(g):
        a = np.ascontiguousarray(og.batch_view(Qd, g, H, s_len * ld, d, s_len, d))
        b = np.ascontiguousarray(og.batch_view(Kd, g, H, s_len * ld, d, s_len, d))
        return og.logical_operands(a, 0, b, 1)
    ph = parts.cpu().numpy()
    ref = oracle_batched(tasks, member, ph, r.numpy(), s.numpy(), 1e-6, True)
    got = tuple(out[k].cpu().numpy() for k in ("lhs", "rhs", "scale")) + (accept.cpu().numpy(),)
    if integer:
        for a, b in zip(got, ref):
            assert np.array_equal(a, b)
    else:
        sizes = np.zeros(n)
        for i, t in enumerate(tasks):
            g = int(t["gemm_id"])
            m0, ml, n0, nl = (int(t[f]) for f in ("m0", "m_len", "n0", "n_len"))
            off = int(t["partial_off"])
            P = np.abs(ph[off:off + ml * nl].astype(np.float64)).reshape(ml, nl)
            sizes[i] = np.abs(r[g].numpy()[m0:m0 + ml]) @ P @ np.abs(s[g].numpy()[n0:n0 + nl])
        compare(tasks, got, ref, sizes)
    assert set(np.flatnonzero(got[3] == 0)) == set(bad)


@pytest.mark.parametrize("transA,transB", [(0, 0), (1, 0), (0, 1)])
def test_verify_grouped_level_matches_oracle(transA, transB):
    """Three same-shape GEMMs of a level (shared A, own B), K-split 2, one pointer per member."""
    M, N, K, tile, S, n = 384, 264, 256, 128, 2, 3
    A_log = make_matrix(71, M, K, "bf16")
    B_logs = [make_matrix(72 + g, K, N, "bf16", std=0.02) for g in range(n)]
    A = stored(A_log, transA)
    Bs = [stored(b, transB) for b in B_logs]
    plan = cleave.plan_batched(M, N, K, tile, tile, S, n)
    tasks, elems = planner.plan_batched(M, N, K, tile, tile, S, n)
    dA, dBs = A.cuda(), [b.cuda() for b in Bs]
    parts = torch.empty(elems, dtype=torch.float32, device="cuda")
    cleave.execute_grouped(plan, [dA] * n, dBs, parts, transA, transB)
    bad = [1, len(tasks) // 2, len(tasks) - 1]
    for i in bad:
        parts[int(tasks[i]["partial_off"]) + 5] -= 500.0
    gen = torch.Generator(device="cpu")
    gen.manual_seed(75)
    r, s = torch.randn((n, M), generator=gen), torch.randn((n, N), generator=gen)
    cnt = plan.num_tasks
    out = {k: torch.full((cnt,), float("nan"), dtype=torch.float64, device="cuda") for k in ("lhs", "rhs", "scale")}
    accept = torch.full((cnt,), -1, dtype=torch.int32, device="cuda")
    cleave.verify_grouped(plan, [dA] * n, dBs, parts, r.cuda(), s.cuda(), 1e-6, accept, out["lhs"], out["rhs"],
                          out["scale"], transA=transA, transB=transB)
    torch.cuda.synchronize()
    ph = parts.cpu().numpy()
    ref = oracle_batched(tasks, lambda g: og.logical_operands(A, transA, Bs[g], transB), ph, r.numpy(), s.numpy(),
                         1e-6, True)
    got = tuple(out[k].cpu().numpy() for k in ("lhs", "rhs", "scale")) + (accept.cpu().numpy(),)
    sizes = np.zeros(cnt)
    for i, t in enumerate(tasks):
        g = int(t["gemm_id"])
        m0, ml, n0, nl = (int(t[f]) for f in ("m0", "m_len", "n0", "n_len"))
        off = int(t["partial_off"])
        P = np.abs(ph[off:off + ml * nl].astype(np.float64)).reshape(ml, nl)
        sizes[i] = np.abs(r[g].numpy()[m0:m0 + ml]) @ P @ np.abs(s[g].numpy()[n0:n0 + nl])
    compare(tasks, got, ref, sizes)
    assert set(np.flatnonzero(got[3] == 0)) == set(bad)
    # plain plans are refused by the batched forms and batched plans by the plain one
    plain = cleave.plan_uniform(M, N, K, tile, tile, S)
    with pytest.raises(cleave.CleaveError):
        cleave.verify_grouped(plain, [dA], dBs[:1], parts, r.cuda(), s.cuda(), 1e-6, accept)
    with pytest.raises(cleave.CleaveError):
        cleave.verify(plan, dA, dBs[0], parts, r.cuda(), s.cuda(), 1e-6, accept, transA=transA, transB=transB)
