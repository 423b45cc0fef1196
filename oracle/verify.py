"""fp64 reference for the random-projection check of returned partial blocks
-- TEST INFRASTRUCTURE ONLY (same rule as the rest of this package).

Sec. 6 "Robustness to poisoning attacks": the parameter server dispatched the
rows of A and the columns of B of a task and receives the block P; for random
vectors r, s it accepts the block when  r^T P s = (A_blk^T r)^T (B_blk s),
which holds exactly for P = A_blk B_blk and costs matrix-vector products only.

With the K-split extension a task's block covers its chunk [k0, k0+k_len) of
the inner dimension, so A_blk is m_len x k_len and B_blk is k_len x n_len.
r has one entry per row of the whole output (a task uses r[m0:m0+m_len]) and s
one per column.

The paper states the identity in exact arithmetic.  In floating point the
two sides differ by rounding; the reading taken here is the standard forward
bound of an inner product: accept iff
    |lhs - rhs| <= tol * scale,   scale = (|r|^T |A_blk|) (|B_blk| |s|),
i.e. the same bilinear form evaluated on absolute values (no cancellation).
All products below are fp64 matrix-vector products of the widened inputs.
"""
import numpy as np


def _ranges(task):
    return (int(task["m0"]), int(task["m_len"]), int(task["n0"]), int(task["n_len"]),
            int(task["k0"]), int(task["k_len"]))


def verify_task(opA, opB, block, task, r, s, tol):
    """Checks one returned block.

    opA (M x K), opB (K x N): fp64 logical operands; block: m_len x n_len values
    of the task's partial block (any float dtype); r (M), s (N): probe vectors.
    Returns (lhs, rhs, scale, accept)."""
    m0, ml, n0, nl, k0, kl = _ranges(task)
    P = np.asarray(block, dtype=np.float64).reshape(ml, nl)
    rb = np.asarray(r[m0:m0 + ml], dtype=np.float64)
    sb = np.asarray(s[n0:n0 + nl], dtype=np.float64)
    A_blk = opA[m0:m0 + ml, k0:k0 + kl]
    B_blk = opB[k0:k0 + kl, n0:n0 + nl]
    lhs = float(rb @ (P @ sb))
    u = A_blk.T @ rb                       # k_len
    v = B_blk @ sb                         # k_len
    rhs = float(u @ v)
    scale = float((np.abs(A_blk).T @ np.abs(rb)) @ (np.abs(B_blk) @ np.abs(sb)))
    accept = abs(lhs - rhs) <= tol * scale
    return lhs, rhs, scale, bool(accept)


def verify_tasks(tasks, opA, opB, partials, r, s, tol):
    """All tasks of a plan against the flat partial buffer.  Returns arrays
    lhs, rhs, scale (fp64) and accept (int32), one entry per task."""
    n = len(tasks)
    lhs = np.zeros(n)
    rhs = np.zeros(n)
    scale = np.zeros(n)
    accept = np.zeros(n, dtype=np.int32)
    for i, t in enumerate(tasks):
        off = int(t["partial_off"])
        cnt = int(t["m_len"]) * int(t["n_len"])
        lhs[i], rhs[i], scale[i], ok = verify_task(opA, opB, partials[off:off + cnt], t, r, s, tol)
        accept[i] = 1 if ok else 0
    return lhs, rhs, scale, accept
