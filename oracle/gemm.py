"""fp64 reference for Cleave's sub-GEMM hot path -- TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's cpu-baseline leg may import
this package; the product path never does.

Definitions followed:
  * a task computes the block of the output given by a set of rows of A and a
    set of columns of B (Sec. 4.1 "Search space of GEMM"); with the K-split
    extension it sums only over its chunk of the inner dimension;
  * the union of the task outputs is the full output and the result equals a
    single-device execution (Sec. 3.2 "Seamless training"), so the reference
    for the final C is the undecomposed fp64 product of the stored inputs;
  * the aggregator sums a tile's S partial blocks in ascending split order;
  * a returned block can be checked with the random-projection identity
    r^T (A B) s = (A^T r)^T (B s) (Sec. 6 "Robustness to poisoning attacks").
"""
import ctypes

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        i64 = ctypes.c_int64
        p = ctypes.c_void_p
        lib.oracle_gemm_f64.argtypes = [i64, i64, i64, i64, p, i64, p, i64, p, i64]
        lib.oracle_gemm_f64.restype = None
        lib.oracle_fold_f32.argtypes = [i64, i64, i64, p, p]
        lib.oracle_fold_f32.restype = None
        lib.oracle_fold_f64.argtypes = [i64, i64, i64, p, p]
        lib.oracle_fold_f64.restype = None
        lib.oracle_num_threads.argtypes = []
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads():
    return int(_load().oracle_num_threads())


def widen(x):
    """Exact widening of stored fp32/bf16 values (torch tensor or ndarray) to fp64."""
    if isinstance(x, np.ndarray):
        return np.ascontiguousarray(x, dtype=np.float64)
    import torch  # the inputs arrive as CPU torch tensors when they are bf16
    return np.ascontiguousarray(x.detach().cpu().to(torch.float64).numpy())


def logical_operands(A, transA, B, transB):
    """Returns fp64 row-major op(A) (M x K) and op(B) (K x N).

    Storage convention of the boundary: transA = 0 -> A is stored M x K,
    transA = 1 -> A is stored K x M; transB = 0 -> B is stored K x N,
    transB = 1 -> B is stored N x K.  The transpose is a layout step only."""
    a = widen(A)
    b = widen(B)
    if transA:
        a = np.ascontiguousarray(a.T)
    if transB:
        b = np.ascontiguousarray(b.T)
    if a.shape[1] != b.shape[0]:
        raise ValueError("inner dimensions differ: %r vs %r" % (a.shape, b.shape))
    return a, b


def gemm(opA, opB, k_begin=0, k_end=None):
    """C = opA[:, k_begin:k_end] @ opB[k_begin:k_end, :] by the naive C loop."""
    M, K = opA.shape
    K2, N = opB.shape
    assert K == K2
    if k_end is None:
        k_end = K
    assert 0 <= k_begin <= k_end <= K
    assert opA.dtype == np.float64 and opB.dtype == np.float64
    assert opA.strides[1] == 8 and opB.strides[1] == 8
    C = np.empty((M, N), dtype=np.float64)
    _load().oracle_gemm_f64(M, N, k_begin, k_end,
                            opA.ctypes.data, opA.strides[0] // 8,
                            opB.ctypes.data, opB.strides[0] // 8,
                            C.ctypes.data, N)
    return C


def task_block(opA, opB, task):
    """fp64 partial block (m_len x n_len) of one task record."""
    m0, ml = int(task["m0"]), int(task["m_len"])
    n0, nl = int(task["n0"]), int(task["n_len"])
    k0, kl = int(task["k0"]), int(task["k_len"])
    rows = opA[m0:m0 + ml, :]                           # alpha rows of A
    cols = np.ascontiguousarray(opB[:, n0:n0 + nl])     # beta columns of B
    return gemm(rows, cols, k0, k0 + kl)


def output_block(opA, opB, m0, m_len, n0, n_len):
    """fp64 block of the undecomposed product (full inner dimension)."""
    rows = opA[m0:m0 + m_len, :]
    cols = np.ascontiguousarray(opB[:, n0:n0 + n_len])
    return gemm(rows, cols)


def execute_tasks(tasks, opA, opB, partial_elems, out=None, task_ids=None):
    """Fills the flat fp64 partial buffer: task t owns
    [partial_off, partial_off + m_len*n_len) as a row-major block."""
    if out is None:
        out = np.zeros(partial_elems, dtype=np.float64)
    ids = range(len(tasks)) if task_ids is None else task_ids
    for i in ids:
        t = tasks[i]
        blk = task_block(opA, opB, t)
        off = int(t["partial_off"])
        out[off:off + blk.size] = blk.reshape(-1)
    return out


def reduce_partials(tasks, partials, M, N):
    """Aggregation: C[tile] = ((P_0 + P_1) + P_2) + ... in ascending split
    order, in the precision of `partials` (fp32 or fp64)."""
    lib = _load()
    if partials.dtype == np.float32:
        fold = lib.oracle_fold_f32
    elif partials.dtype == np.float64:
        fold = lib.oracle_fold_f64
    else:
        raise TypeError(partials.dtype)
    assert partials.flags["C_CONTIGUOUS"]
    C = np.zeros((M, N), dtype=partials.dtype)
    item = partials.dtype.itemsize
    for t in tasks:
        if int(t["ksplit_idx"]) != 0:
            continue
        S = int(t["ksplit_cnt"])
        ml, nl = int(t["m_len"]), int(t["n_len"])
        m0, n0 = int(t["m0"]), int(t["n0"])
        off = int(t["partial_off"])
        cnt = ml * nl
        blk = np.empty(cnt, dtype=partials.dtype)
        fold(S, cnt, cnt, partials.ctypes.data + off * item, blk.ctypes.data)
        C[m0:m0 + ml, n0:n0 + nl] = blk.reshape(ml, nl)
    return C


def batch_view(stored, g, n_inner, outer_stride, inner_stride, rows, cols):
    """Zero-copy view of GEMM g's stored operand inside a larger 2-D array:
    g = o * n_inner + i starts at flat element o * outer_stride + i * inner_stride
    of `stored` (row-major, leading dimension = its row length) and spans
    rows x cols with the same leading dimension -- the boundary's batch
    convention.  Returns an ndarray view (no arithmetic)."""
    ld = stored.shape[1]
    o, i = divmod(g, n_inner)
    start = o * outer_stride + i * inner_stride
    flat = stored.reshape(-1)
    span = (rows - 1) * ld + cols
    if start < 0 or start + span > flat.size:
        raise ValueError("batch view out of range")
    return np.lib.stride_tricks.as_strided(flat[start:], shape=(rows, cols),
                                           strides=(ld * flat.itemsize, flat.itemsize), writeable=False)


def rel_frobenius(C, C_ref):
    """||C - C_ref||_F / ||C_ref||_F in fp64."""
    c = np.asarray(C, dtype=np.float64)
    r = np.asarray(C_ref, dtype=np.float64)
    den = np.linalg.norm(r)
    return float(np.linalg.norm(c - r) / den) if den > 0 else float(np.linalg.norm(c - r))


def projection_check(opA, opB, C, seed):
    """Random-projection identity of Sec. 6 ("Robustness to poisoning
    attacks"): returns |r^T C s - (A^T r)^T (B s)| divided by the size scale
    ||r||*||C s|| so that rounding noise reads as ~1e-16..1e-7 and a wrong
    block as O(1e-3) or more.  fp64 matrix-vector products only."""
    rng = np.random.default_rng(seed)
    M, N = C.shape
    r = rng.standard_normal(M)
    s = rng.standard_normal(N)
    Cs = np.asarray(C, dtype=np.float64) @ s
    lhs = float(r @ Cs)
    rhs = float((opA.T @ r) @ (opB @ s))
    scale = float(np.linalg.norm(r) * np.linalg.norm(Cs)) or 1.0
    return abs(lhs - rhs) / scale
