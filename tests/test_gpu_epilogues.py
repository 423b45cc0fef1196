"""GPU parity of the aggregation epilogues (residual add, Adam update) against
their fp64 oracle.  The partial blocks are seeded random fp32 values; the
aggregated value both sides start from is the fp32 left fold, which the reduce
tests pin bitwise, so the oracle folds the same partials with its own fold and
applies the operator in fp64.

Bars: fp32 results within a few units in the last place of the fp64 result
(the GPU evaluates the same formula in fp32 with correctly rounded division and
square root); the bf16 copy of a weight is the round-to-nearest-even of the
GPU's own fp32 weight, bit for bit (the rounding decision is taken in the same
precision on both sides).
"""
import numpy as np
import pytest
import torch

import paper_2512_22142_amd as cleave
from oracle import gemm as og
from oracle import optimizer as oo
from oracle import planner

pytestmark = pytest.mark.gpu

EPS32 = 2.0 ** -24

SHAPES = [(256, 384, 128, 128, 4), (300, 200, 128, 128, 2), (37, 29, 16, 8, 3), (640, 392, 256, 256, 1)]


def f32(x):
    """The fp32 value the C ABI receives for a hyper-parameter, as a Python float:
    both sides then work from the same numbers."""
    return float(np.float32(x))


def seeded(shape, seed, scale=1.0):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return torch.randn(shape, generator=g, dtype=torch.float32) * scale


def folded(tasks, parts, M, N):
    return og.reduce_partials(tasks, parts, M, N)          # fp32 left fold (oracle's own)


@pytest.mark.parametrize("M,N,tm,tn,S", SHAPES)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_reduce_residual_matches_oracle(M, N, tm, tn, S, dtype):
    K = 64
    plan = cleave.plan_uniform(M, N, K, tm, tn, S)
    tasks, elems = planner.plan_uniform(M, N, K, tm, tn, S)
    parts = seeded((elems,), 101 + M)
    R = seeded((M, N), 102 + N).to(dtype)
    C = torch.full((M, N), float("nan"), dtype=dtype, device="cuda")
    cleave.reduce_residual(plan, parts.cuda(), R.cuda(), C)
    torch.cuda.synchronize()
    fold = folded(tasks, parts.numpy(), M, N)
    ref = oo.add_residual(fold, R.to(torch.float32).numpy())
    got = C.to(torch.float32).cpu().numpy().astype(np.float64)
    ulp = (2.0 ** -8 if dtype == torch.bfloat16 else EPS32) * np.abs(ref) + 1e-38
    assert np.all(np.abs(got - ref) <= ulp * (1 + 1e-6))
    # the fp32 sum is one IEEE add; the bf16 result its nearest-even rounding
    one_add = fold + R.to(torch.float32).numpy()
    expect = oo.bf16_round(one_add) if dtype == torch.bfloat16 else one_add
    assert np.array_equal(C.to(torch.float32).cpu().numpy(), expect)
    # in place: R is the output
    Rd = R.cuda()
    cleave.reduce_residual(plan, parts.cuda(), Rd, Rd)
    torch.cuda.synchronize()
    assert torch.equal(Rd, C)


def adam_bounds(w_old, m_old, v_old, g, h, step):
    """Rounding bounds of the fp32 evaluation of one update, derived from its
    formula: the moments are two products and a sum; the weight step is
    lr * mhat / (sqrt(vhat) + eps), whose error is the moments' errors pushed
    through that quotient plus a few roundings of its own."""
    b1, b2 = h["beta1"], h["beta2"]
    m_b = 4 * EPS32 * (np.abs(b1 * m_old) + np.abs((1 - b1) * g)) + 1e-44
    v_b = 6 * EPS32 * (np.abs(b2 * v_old) + (1 - b2) * g * g) + 1e-44
    ib1, ib2 = 1 / (1 - b1 ** step), 1 / (1 - b2 ** step)
    mh = (b1 * m_old + (1 - b1) * g) * ib1
    vh = (b2 * v_old + (1 - b2) * g * g) * ib2
    den = np.sqrt(vh) + h["eps"]
    u = np.abs(mh) / den
    du = m_b * ib1 / den + u * (v_b * ib2) / (2 * np.sqrt(vh) * den + 1e-300) + 8 * EPS32 * u
    w_b = 2 * EPS32 * np.abs(w_old) + h["lr"] * (du + 4 * EPS32 * h["weight_decay"] * np.abs(w_old)) + 1e-12
    return m_b, v_b, w_b


@pytest.mark.parametrize("M,N,tm,tn,S", SHAPES)
@pytest.mark.parametrize("wd,with_copy", [(0.0, True), (0.01, False)])
def test_reduce_adam_matches_oracle(M, N, tm, tn, S, wd, with_copy):
    """One update from a given state, at three points of a run: the first step
    (zero moments) and later steps with seeded moments.  Each case starts both
    sides from the same seeded state, so no error carries over."""
    K = 64
    h = dict(lr=f32(1e-3), beta1=f32(0.9), beta2=f32(0.95), eps=f32(1e-8), weight_decay=f32(wd))
    plan = cleave.plan_uniform(M, N, K, tm, tn, S)
    tasks, elems = planner.plan_uniform(M, N, K, tm, tn, S)
    for step in (1, 2, 50):
        parts = seeded((elems,), 120 + step, 0.5)
        w0 = seeded((M, N), 111 + step, 0.02)
        m0 = torch.zeros(M, N) if step == 1 else seeded((M, N), 112 + step, 0.3)
        v0 = torch.zeros(M, N) if step == 1 else seeded((M, N), 113 + step, 0.3).abs()
        w, m, v = w0.cuda(), m0.cuda(), v0.cuda()
        w16 = torch.zeros(M, N, dtype=torch.bfloat16, device="cuda") if with_copy else None
        cleave.reduce_adam(plan, parts.cuda(), w, m, v, step=step, w_bf16=w16, **h)
        torch.cuda.synchronize()
        g = folded(tasks, parts.numpy(), M, N).astype(np.float64)
        wr, mr, vr = (x.numpy().astype(np.float64) for x in (w0, m0, v0))
        m_b, v_b, w_b = adam_bounds(wr, mr, vr, g, h, step)
        wr, mr, vr = oo.adam_step(wr, mr, vr, g, step=step, **h)
        wg, mg, vg = (x.cpu().numpy().astype(np.float64) for x in (w, m, v))
        assert np.all(np.abs(mg - mr) <= m_b), step
        assert np.all(np.abs(vg - vr) <= v_b), step
        assert np.all(np.abs(wg - wr) <= w_b), step
        if with_copy:
            assert np.array_equal(w16.to(torch.float32).cpu().numpy(), oo.bf16_round(w.cpu().numpy()))


def test_reduce_adam_first_step_moves_by_lr_and_zero_gradient_keeps_weights():
    M, N, K = 128, 128, 64
    plan = cleave.plan_uniform(M, N, K, 64, 64, 2)
    parts = seeded((plan.partial_elems,), 131)
    w = seeded((M, N), 132).cuda()
    w_before = w.clone()
    m, v = torch.zeros(M, N, device="cuda"), torch.zeros(M, N, device="cuda")
    cleave.reduce_adam(plan, parts.cuda(), w, m, v, 1e-3, 0.9, 0.999, 0.0, 0.0, 1)
    torch.cuda.synchronize()
    moved = (w - w_before).abs().cpu().numpy()
    assert np.all(np.abs(moved - 1e-3) <= 2e-7 + 2 * EPS32 * np.abs(w_before.cpu().numpy()))
    z = torch.zeros(plan.partial_elems, device="cuda")
    w2, m2, v2 = w.clone(), torch.zeros(M, N, device="cuda"), torch.zeros(M, N, device="cuda")
    cleave.reduce_adam(plan, z, w2, m2, v2, 1e-3, 0.9, 0.999, 1e-8, 0.0, 4)
    torch.cuda.synchronize()
    assert torch.equal(w2, w) and not m2.any() and not v2.any()


def test_reduce_adam_at_a_llama7b_weight_gradient():
    """gate.dw of the c3 layer: 4096 x 11008 weight, 512 x 512 tiles, S = 4."""
    M, N, K, S = 4096, 11008, 4096, 4
    h = dict(lr=f32(3e-4), beta1=f32(0.9), beta2=f32(0.95), eps=f32(1e-8), weight_decay=f32(0.1))
    plan = cleave.plan_uniform(M, N, K, 512, 512, S)
    tasks, elems = planner.plan_uniform(M, N, K, 512, 512, S)
    parts = seeded((elems,), 141, 0.1)
    w0, m0, v0 = seeded((M, N), 142, 0.02), seeded((M, N), 143, 0.01), seeded((M, N), 144, 0.01).abs()
    w, m, v = w0.cuda(), m0.cuda(), v0.cuda()
    w16 = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    cleave.reduce_adam(plan, parts.cuda(), w, m, v, step=9, w_bf16=w16, **h)
    torch.cuda.synchronize()
    g = folded(tasks, parts.numpy(), M, N).astype(np.float64)
    wr, mr, vr = oo.adam_step(w0.numpy(), m0.numpy(), v0.numpy(), g, step=9, **h)
    m_b, v_b, w_b = adam_bounds(w0.numpy().astype(np.float64), m0.numpy().astype(np.float64),
                                v0.numpy().astype(np.float64), g, h, 9)
    wg = w.cpu().numpy()
    assert np.all(np.abs(m.cpu().numpy() - mr) <= m_b) and np.all(np.abs(v.cpu().numpy() - vr) <= v_b)
    assert np.all(np.abs(wg - wr) <= w_b)
    assert np.array_equal(w16.to(torch.float32).cpu().numpy(), oo.bf16_round(wg))


def test_epilogues_reject_bad_arguments():
    plan = cleave.plan_uniform(64, 64, 64, 32, 32, 1)
    parts = torch.zeros(plan.partial_elems, device="cuda")
    w = torch.zeros(64, 64, device="cuda")
    for kw in (dict(step=0), dict(beta1=1.0), dict(beta2=-0.1), dict(eps=-1.0), dict(lr=float("nan"))):
        a = dict(lr=1e-3, beta1=0.9, beta2=0.99, eps=1e-8, weight_decay=0.0, step=1)
        a.update(kw)
        with pytest.raises(cleave.CleaveError):
            cleave.reduce_adam(plan, parts, w, w.clone(), w.clone(), **a)
    bp = cleave.plan_batched(64, 64, 64, 32, 32, 1, 2)
    with pytest.raises(cleave.CleaveError):
        cleave.reduce_residual(bp, torch.zeros(bp.partial_elems, device="cuda"), w, w)


@pytest.mark.parametrize("M,N,tm,tn,S,n", [(256, 384, 128, 128, 4, 3), (300, 200, 128, 128, 2, 2), (37, 29, 16, 8, 3, 4)])
def test_grouped_adam_equals_the_single_calls_bit_for_bit(M, N, tm, tn, S, n):
    """The weight-gradient GEMMs of a level in one launch: member g's weight, moments
    and bf16 copy come out exactly as the single-GEMM call leaves them (whose result
    the tests above hold against the fp64 oracle)."""
    K = 64
    single = cleave.plan_uniform(M, N, K, tm, tn, S)
    group = cleave.plan_batched(M, N, K, tm, tn, S, n)
    assert group.partial_elems == n * single.partial_elems
    parts = seeded((group.partial_elems,), 900 + M).cuda()
    hyper = (f32(1e-3), f32(0.9), f32(0.95), f32(1e-8), f32(0.1))
    w0 = [seeded((M, N), 910 + g, 0.02) for g in range(n)]
    m0 = [seeded((M, N), 920 + g, 0.01) for g in range(n)]
    v0 = [seeded((M, N), 930 + g, 0.01).abs() for g in range(n)]
    # grouped: three steps in a row
    gw, gm, gv = [t.clone().cuda() for t in w0], [t.clone().cuda() for t in m0], [t.clone().cuda() for t in v0]
    gb = [torch.empty((M, N), dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    for step in (1, 2, 3):
        cleave.reduce_adam_grouped(group, parts, gw, gm, gv, *hyper, step, w_bf16_list=gb)
    # single calls on each member's slice of the partial buffer
    for g in range(n):
        sw, sm, sv = w0[g].clone().cuda(), m0[g].clone().cuda(), v0[g].clone().cuda()
        sb = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        mine = parts[g * single.partial_elems:(g + 1) * single.partial_elems]
        for step in (1, 2, 3):
            cleave.reduce_adam(single, mine, sw, sm, sv, *hyper, step, w_bf16=sb)
        torch.cuda.synchronize()
        for got, want in ((gw[g], sw), (gm[g], sm), (gv[g], sv)):
            assert torch.equal(got.view(torch.int32), want.view(torch.int32)), g
        assert torch.equal(gb[g].view(torch.int16), sb.view(torch.int16)), g
    # without bf16 copies, and argument checks
    cleave.reduce_adam_grouped(group, parts, gw, gm, gv, *hyper, 4)
    with pytest.raises(cleave.CleaveError):
        cleave.reduce_adam_grouped(single, parts, gw[:1], gm[:1], gv[:1], *hyper, 1)      # plain plan
    with pytest.raises(cleave.CleaveError):
        cleave.reduce_adam_grouped(group, parts, gw[:-1], gm[:-1], gv[:-1], *hyper, 1)    # one member short
    with pytest.raises(cleave.CleaveError):
        cleave.reduce_adam_grouped(group, parts, gw, gm, gv, *hyper, 0)                   # steps count from 1
