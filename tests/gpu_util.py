"""Helpers of the GPU parity tests: run plan/execute/reduce through the C ABI
on device copies of CPU tensors and fetch results back."""
import numpy as np
import torch

import paper_2512_22142_amd as cleave

TOL = {"f32": 1e-5, "bf16": 5e-3}    # relative Frobenius bound per input type


def stored(logical, trans):
    """CPU tensor holding `logical` (M x K or K x N) in the boundary's stored
    layout: as is, or as its transpose when trans = 1."""
    return logical.t().contiguous() if trans else logical.contiguous()


class GpuGemm:
    """One GEMM on the GPU: owns device operands, partial buffer and C."""

    def __init__(self, plan, A_cpu, B_cpu, transA=0, transB=0, out_dtype=torch.float32):
        self.plan = plan
        self.transA, self.transB = transA, transB
        self.A = A_cpu.cuda()
        self.B = B_cpu.cuda()
        self.partials = torch.empty(plan.partial_elems, dtype=torch.float32, device="cuda")
        self.C = torch.empty((plan.M, plan.N), dtype=out_dtype, device="cuda")

    def execute(self, task_ids=None):
        cleave.execute(self.plan, self.A, self.B, self.partials, self.transA, self.transB,
                       task_ids=task_ids)
        return self

    def reduce(self):
        cleave.reduce(self.plan, self.partials, self.C)
        return self

    def run(self):
        return self.execute().reduce()

    def C_host(self):
        torch.cuda.synchronize()
        return self.C.float().cpu().numpy()

    def partials_host(self):
        torch.cuda.synchronize()
        return self.partials.cpu().numpy()


def block_of(partials, task):
    off = int(task["partial_off"])
    ml, nl = int(task["m_len"]), int(task["n_len"])
    return partials[off:off + ml * nl].reshape(ml, nl)


def elementwise_bound(rows, cols, k0, k1):
    """Per-element bound on |fp32-accumulated block - fp64 block| for the block
    rows[:, k0:k1] @ cols[k0:k1, :] of exactly representable inputs (products
    of bf16 values are exact in fp32, so only the K additions round):

        |err_ij| <= 8 * 2^-24 * ||a_i||_2 * ||b_j||_2      (norms over the chunk)

    Rounding errors of a length-K fp32 accumulation add up like a random walk
    over partial sums of size ~ sqrt(k) * rms(a) * rms(b); their standard
    deviation is about 2^-24 * ||a_i|| * ||b_j|| / sqrt(2), so this is an
    11-sigma bound (and far inside the deterministic K * 2^-24 * sum |a||b|).
    Relative to the size of an output element it is ~5e-7 * sqrt(K): an
    element wrong in its fifth digit fails, wherever it is."""
    na = np.linalg.norm(rows[:, k0:k1], axis=1)
    nb = np.linalg.norm(cols[k0:k1, :], axis=0)
    return 8.0 * 2.0 ** -24 * np.outer(na, nb)


def assert_elementwise(got, ref, bound, what):
    """got (fp32 from the GPU) against ref (fp64 from the oracle), element by
    element, plus the regression bar of 1e-5 in the Frobenius norm."""
    diff = np.abs(got.astype(np.float64) - ref)
    worst = np.argmax(diff - bound)
    assert np.all(diff <= bound), (what, np.unravel_index(worst, diff.shape),
                                   float(diff.reshape(-1)[worst]), float(bound.reshape(-1)[worst]))
    den = np.linalg.norm(ref)
    assert den == 0 or np.linalg.norm(diff) / den <= 1e-5, what
