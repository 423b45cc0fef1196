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
