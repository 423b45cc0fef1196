"""The persistent multi-item path of the direct bf16 kernel, bit for bit.

Every workgroup here runs several short work items in a row (more than twice
as many items as the chip holds workgroups), so the code between two items is
what is tested: the next item's ring fill issued ahead of the current item's
stores, the shortened wait that relies on those stores, the item record
fetched during the epilogue, the fall-back wait after a clipped (ragged)
sub-tile followed again by full ones.  Chunks of 1, 2 and 3 K steps keep the
K loop short, so nearly all of a launch is that code.  Integer-valued inputs:
every partial block and the whole of C must equal the fp64 oracle exactly.
"""
import numpy as np
import pytest
import torch

import paper_2512_22142_amd as cleave
from oracle import gemm as og
from oracle import planner
from workloads.tensors import make_matrix

from gpu_util import GpuGemm, block_of, stored

pytestmark = pytest.mark.gpu

LAYOUTS = [(0, 0), (0, 1), (1, 0), (1, 1)]
K_STEP = 64          # elements of K the direct kernel consumes per step


def _resident_workgroups(per_cu):
    return torch.cuda.get_device_properties(0).multi_processor_count * per_cu


@pytest.mark.parametrize("transA,transB", LAYOUTS)
@pytest.mark.parametrize("steps", [1, 2, 3])
@pytest.mark.parametrize("cls", ["large", "small"])
def test_many_short_items_per_workgroup_exact(cls, steps, transA, transB):
    S = 2
    K = K_STEP * steps * S
    if cls == "large":
        # 384 x 384 tiles are cut into a full 256 x 256 sub-tile and three clipped ones
        # (256 x 128, 128 x 256, 128 x 128), so full and clipped items alternate in every
        # workgroup; the last 40 columns form narrow tiles of the small class
        M, N, tile = 6144, 4264, 384
        per_cu, sub = 1, 256
    else:
        M, N, tile = 4160, 4104, 128
        per_cu, sub = 2, 128
    n_items = -(-M // sub) * -(-N // sub) * S
    assert n_items > 2 * _resident_workgroups(per_cu), "the shape must give every workgroup several items"
    a = make_matrix(500 + steps, M, K, "bf16", integer_valued=True)
    b = make_matrix(600 + steps, K, N, "bf16", integer_valued=True)
    plan = cleave.plan_uniform(M, N, K, tile, tile, S)
    tasks, _ = planner.plan_uniform(M, N, K, tile, tile, S)
    assert plan.tasks.tobytes() == tasks.tobytes()
    run = GpuGemm(plan, stored(a, transA), stored(b, transB), transA, transB).run()
    assert "direct" in plan.last_kernel and ("256x256" if cls == "large" else "128x128") in plan.last_kernel
    parts, C = run.partials_host(), run.C_host()
    opA, opB = og.logical_operands(stored(a, transA), transA, stored(b, transB), transB)
    total = np.zeros((M, N))
    for s in range(S):
        ref = og.gemm(opA, opB, s * K // S, (s + 1) * K // S)
        for t in tasks[tasks["ksplit_idx"] == s]:
            m0, ml, n0, nl = int(t["m0"]), int(t["m_len"]), int(t["n0"]), int(t["n_len"])
            assert np.array_equal(block_of(parts, t), ref[m0:m0 + ml, n0:n0 + nl]), (int(t["tile_id"]), s)
        total += ref
    assert np.array_equal(C, total)


@pytest.mark.parametrize("out", ["partials", "assembled_f32", "assembled_bf16"])
def test_outputs_that_only_take_element_stores_exact(out):
    """The fast kernel writes full sub-tiles with 16-byte stores when the output
    allows them.  Here it does not: the partial workspace starts one element
    into its allocation, the assembled output has an odd row pitch and starts
    one element in.  Same kernel, element stores, several items per workgroup,
    every value equal to the oracle's."""
    M, N, tile = 8192, 4096, 256
    S = 4 if out == "partials" else 1
    K = 2 * K_STEP * S
    assert (M // tile) * (N // tile) * S >= 2 * _resident_workgroups(1)
    a = make_matrix(701, M, K, "bf16", integer_valued=True)
    b = make_matrix(702, K, N, "bf16", integer_valued=True)
    plan = cleave.plan_uniform(M, N, K, tile, tile, S)
    tasks, elems = planner.plan_uniform(M, N, K, tile, tile, S)
    dA, dB = a.cuda(), b.cuda()
    opA, opB = og.logical_operands(a, 0, b, 0)
    ref = og.gemm(opA, opB)
    if out == "partials":
        raw = torch.full((elems + 1,), float("nan"), dtype=torch.float32, device="cuda")
        parts = raw[1:]
        assert parts.data_ptr() % 16 == 4
        cleave.execute(plan, dA, dB, parts)
        assert "direct" in plan.last_kernel
        torch.cuda.synchronize()
        host = parts.cpu().numpy()
        for s in range(S):
            ref_s = og.gemm(opA, opB, s * K // S, (s + 1) * K // S)
            for t in tasks[tasks["ksplit_idx"] == s]:
                m0, ml, n0, nl = int(t["m0"]), int(t["m_len"]), int(t["n0"]), int(t["n_len"])
                assert np.array_equal(block_of(host, t), ref_s[m0:m0 + ml, n0:n0 + nl]), (int(t["tile_id"]), s)
        assert np.isnan(raw[:1].cpu().numpy()).all()
    else:
        dt = torch.float32 if out == "assembled_f32" else torch.bfloat16
        wide = torch.full((M, N + 3), float("nan"), dtype=dt, device="cuda")
        C = wide[:, 1:N + 1]
        cleave.execute_assemble(plan, dA, dB, C)
        assert "direct" in plan.last_kernel
        torch.cuda.synchronize()
        got = C.float().cpu().numpy()
        want = ref if dt == torch.float32 else torch.from_numpy(ref).to(torch.bfloat16).float().numpy()
        assert np.array_equal(got, want)
        pad = torch.cat([wide[:, :1], wide[:, N + 1:]], dim=1).float().cpu().numpy()
        assert np.isnan(pad).all()          # nothing written outside the view


@pytest.mark.parametrize("transA,transB", [(0, 0), (0, 1), (1, 0)])
def test_items_of_unequal_length_take_the_balanced_schedule_exact(transA, transB):
    """Tiles with 1, 2, 4 and 8 splits of the inner dimension in one plan: chunk
    lengths differ by a factor of eight, so the library gives every workgroup a
    run of items of its own (longest items placed first) instead of every
    grid-th item.  Several items per workgroup; every block and C exact."""
    M, N, K = 4096, 6144, 512
    band_h = [512] * 8
    col_w = [[512] * 12 for _ in band_h]
    ks = [(1, 2, 4, 8)[(3 * i + j) % 4] for i in range(8) for j in range(12)]
    plan = cleave.plan_explicit(M, N, K, band_h, col_w, ks)
    tasks, _ = planner.plan_explicit(M, N, K, band_h, col_w, ks)
    assert plan.tasks.tobytes() == tasks.tobytes()
    # every task is a 512 x 512 block: four 256 x 256 work items
    assert 4 * len(tasks) > 2 * _resident_workgroups(1)
    a = make_matrix(801, M, K, "bf16", integer_valued=True)
    b = make_matrix(802, K, N, "bf16", integer_valued=True)
    run = GpuGemm(plan, stored(a, transA), stored(b, transB), transA, transB).run()
    assert "direct" in plan.last_kernel
    parts, C = run.partials_host(), run.C_host()
    opA, opB = og.logical_operands(stored(a, transA), transA, stored(b, transB), transB)
    bounds = sorted(set((int(t["k0"]), int(t["k0"]) + int(t["k_len"])) for t in tasks))
    ref_of = {kb: og.gemm(opA, opB, kb[0], kb[1]) for kb in bounds}
    for t in tasks:
        m0, ml, n0, nl = int(t["m0"]), int(t["m_len"]), int(t["n0"]), int(t["n_len"])
        ref = ref_of[(int(t["k0"]), int(t["k0"]) + int(t["k_len"]))]
        assert np.array_equal(block_of(parts, t), ref[m0:m0 + ml, n0:n0 + nl]), (int(t["tile_id"]), int(t["ksplit_idx"]))
    assert np.array_equal(C, og.gemm(opA, opB))
    # a re-issued subset goes the unbalanced way (its list is made on the device): same bits
    ids = [int(i) for i in range(0, len(tasks), 7)]
    run.partials[:] = float("nan")
    run.execute(task_ids=ids)
    again = run.partials_host()
    for i in ids:
        assert np.array_equal(block_of(again, tasks[i]), block_of(parts, tasks[i]))
