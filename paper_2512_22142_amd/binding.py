"""ctypes binding of libcleave.so: argument marshalling only.

Every step of the path (task generation, sub-GEMM execution, aggregation) runs
inside the library; torch tensors are used here solely as owners of device
memory and as the source of the current HIP stream.  There is no fallback: if
the library has not been built, importing this module raises.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcleave.so")

F32 = 0
BF16 = 1

OK, EINVAL, ENOMEM, EHIP, ELIMIT = 0, -1, -2, -3, -4

# Byte layout of `cleave_task` (include/cleave.h).
TASK_DTYPE = np.dtype([
    ("gemm_id", "<u4"), ("tile_id", "<u4"),
    ("m0", "<u4"), ("m_len", "<u4"), ("n0", "<u4"), ("n_len", "<u4"),
    ("k0", "<u4"), ("k_len", "<u4"),
    ("ksplit_idx", "<u4"), ("ksplit_cnt", "<u4"),
    ("partial_off", "<u8"),
    ("flags", "<u4"), ("reserved", "<u4", (3,)),
])
assert TASK_DTYPE.itemsize == 64

EXPORTS = (
    "cleave_plan_uniform", "cleave_plan_explicit", "cleave_plan_num_tasks",
    "cleave_plan_num_tiles", "cleave_plan_tasks", "cleave_plan_partial_elems",
    "cleave_plan_dims", "cleave_plan_upload", "cleave_plan_destroy", "cleave_execute",
    "cleave_reduce", "cleave_strerror", "cleave_last_hip_error", "cleave_version",
    "cleave_plan_last_kernel", "cleave_verify", "cleave_plan_batched", "cleave_execute_batched",
    "cleave_reduce_batched", "cleave_reduce_residual", "cleave_reduce_adam",
    "cleave_shard_cost", "cleave_shard_fits", "cleave_assign", "cleave_reassign", "cleave_execute_assemble",
    "cleave_execute_grouped", "cleave_reduce_grouped", "cleave_execute_noalloc", "cleave_reassign_sets", "cleave_reduce_adam_grouped", "cleave_verify_batched", "cleave_verify_grouped", "cleave_verify_reduce", "cleave_plan_schedule_loads",
)


class Device(ctypes.Structure):
    """cleave_device: bytes/s, s, flop/s, bytes."""
    _fields_ = [("down_bw", ctypes.c_double), ("up_bw", ctypes.c_double),
                ("down_lat", ctypes.c_double), ("up_lat", ctypes.c_double),
                ("flops", ctypes.c_double), ("mem_bytes", ctypes.c_double)]


class CleaveError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = _lib.cleave_strerror(status).decode()
        if status == EHIP:
            msg += " (hipError_t %d)" % _lib.cleave_last_hip_error()
        super().__init__("%s: %s" % (where, msg))


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libcleave.so is not built: run `python -m paper_2512_22142_amd.build` "
            "(or __graft_entry__.build()) first")
    # Device pointers and streams come from PyTorch, so the library must bind to
    # the HIP runtime instance PyTorch has loaded: import torch first, whatever
    # order the caller imports things in (two runtimes in one process do not see
    # each other's devices or allocations).
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    i64, i32, u32, p = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32, ctypes.c_void_p
    lib.cleave_plan_uniform.argtypes = [i64, i64, i64, i64, i64, i32, u32, ctypes.POINTER(p)]
    lib.cleave_plan_uniform.restype = ctypes.c_int
    lib.cleave_plan_explicit.argtypes = [i64, i64, i64, i32, p, p, p, p, u32, ctypes.POINTER(p)]
    lib.cleave_plan_explicit.restype = ctypes.c_int
    for name in ("cleave_plan_num_tasks", "cleave_plan_num_tiles", "cleave_plan_partial_elems"):
        getattr(lib, name).argtypes = [p]
        getattr(lib, name).restype = i64
    lib.cleave_plan_tasks.argtypes = [p]
    lib.cleave_plan_tasks.restype = p
    lib.cleave_plan_dims.argtypes = [p, p]
    lib.cleave_plan_dims.restype = ctypes.c_int
    lib.cleave_plan_upload.argtypes = [p]
    lib.cleave_plan_upload.restype = ctypes.c_int
    lib.cleave_plan_destroy.argtypes = [p]
    lib.cleave_plan_destroy.restype = None
    lib.cleave_execute.argtypes = [p, p, i64, p, i64, ctypes.c_int, p, i64, ctypes.c_int,
                                   ctypes.c_int, p, p]
    lib.cleave_execute.restype = ctypes.c_int
    lib.cleave_execute_noalloc.argtypes = lib.cleave_execute.argtypes
    lib.cleave_execute_noalloc.restype = ctypes.c_int
    lib.cleave_reduce.argtypes = [p, p, p, i64, ctypes.c_int, p]
    lib.cleave_plan_batched.argtypes = [i64, i64, i64, i64, i64, i32, i64, ctypes.POINTER(p)]
    lib.cleave_plan_batched.restype = ctypes.c_int
    lib.cleave_execute_batched.argtypes = [p, p, i64, p, i64, ctypes.c_int, i64, i64,
                                           p, i64, ctypes.c_int, i64, i64, i64, ctypes.c_int, p, p]
    lib.cleave_execute_batched.restype = ctypes.c_int
    lib.cleave_execute_assemble.argtypes = [p, p, i64, p, i64, ctypes.c_int, i64, i64,
                                            p, i64, ctypes.c_int, i64, i64, i64, ctypes.c_int,
                                            p, i64, i64, i64, ctypes.c_int, p]
    lib.cleave_execute_assemble.restype = ctypes.c_int
    lib.cleave_reduce_batched.argtypes = [p, p, p, i64, i64, i64, i64, ctypes.c_int, p]
    lib.cleave_reduce_batched.restype = ctypes.c_int
    lib.cleave_execute_grouped.argtypes = [p, p, i64, i64, p, i64, ctypes.c_int, p, i64, ctypes.c_int,
                                           ctypes.c_int, p, p]
    lib.cleave_execute_grouped.restype = ctypes.c_int
    lib.cleave_reduce_grouped.argtypes = [p, p, i64, p, i64, ctypes.c_int, p]
    lib.cleave_reduce_grouped.restype = ctypes.c_int
    lib.cleave_reduce_residual.argtypes = [p, p, p, p, i64, ctypes.c_int, p]
    lib.cleave_reduce_residual.restype = ctypes.c_int
    f32 = ctypes.c_float
    lib.cleave_reduce_adam.argtypes = [p, p, p, p, p, p, i64, f32, f32, f32, f32, f32, i64, p]
    lib.cleave_reduce_adam.restype = ctypes.c_int
    lib.cleave_reduce_adam_grouped.argtypes = [p, p, i64, p, p, p, p, i64, f32, f32, f32, f32, f32, i64, p]
    lib.cleave_reduce_adam_grouped.restype = ctypes.c_int
    lib.cleave_shard_cost.argtypes = [p, i64, i64, i64, i64, i64, i32]
    lib.cleave_shard_cost.restype = ctypes.c_double
    lib.cleave_shard_fits.argtypes = [p, i64, i64, i64, i32]
    lib.cleave_shard_fits.restype = ctypes.c_int
    lib.cleave_assign.argtypes = [i64, i64, i64, i32, p, i32, i64, p, p, p, p, p, p]
    lib.cleave_assign.restype = ctypes.c_int
    lib.cleave_reassign.argtypes = [i64, i64, i64, i32, p, i32, i64, i64, i64, p, p, p, p, p, p, p, p]
    lib.cleave_reassign.restype = ctypes.c_int
    lib.cleave_reassign_sets.argtypes = [i64, i64, i64, i32, p, i32, i64, i64, i64, p, p, p, p, p, p, p, p, p, p, p]
    lib.cleave_reassign_sets.restype = ctypes.c_int
    lib.cleave_verify.argtypes = [p, p, i64, ctypes.c_int, p, i64, ctypes.c_int, ctypes.c_int,
                                  p, p, p, ctypes.c_double, p, p, p, p, p]
    lib.cleave_verify.restype = ctypes.c_int
    lib.cleave_plan_schedule_loads.argtypes = [p, ctypes.c_int, ctypes.c_int, ctypes.c_int, p]
    lib.cleave_plan_schedule_loads.restype = ctypes.c_int
    lib.cleave_verify_reduce.argtypes = [p, p, i64, ctypes.c_int, p, i64, ctypes.c_int, ctypes.c_int,
                                         p, p, p, ctypes.c_double, p, p, p, p, p, i64, ctypes.c_int, p]
    lib.cleave_verify_reduce.restype = ctypes.c_int
    lib.cleave_verify_batched.argtypes = [p, p, i64, ctypes.c_int, i64, i64, p, i64, ctypes.c_int, i64, i64, i64,
                                          ctypes.c_int, p, p, p, ctypes.c_double, p, p, p, p, p]
    lib.cleave_verify_batched.restype = ctypes.c_int
    lib.cleave_verify_grouped.argtypes = [p, i64, p, i64, ctypes.c_int, p, i64, ctypes.c_int, ctypes.c_int,
                                          p, p, p, ctypes.c_double, p, p, p, p, p]
    lib.cleave_verify_grouped.restype = ctypes.c_int
    lib.cleave_reduce.restype = ctypes.c_int
    lib.cleave_strerror.argtypes = [ctypes.c_int]
    lib.cleave_strerror.restype = ctypes.c_char_p
    lib.cleave_last_hip_error.argtypes = []
    lib.cleave_last_hip_error.restype = ctypes.c_int
    lib.cleave_version.argtypes = []
    lib.cleave_version.restype = ctypes.c_int
    lib.cleave_plan_last_kernel.argtypes = [p]
    lib.cleave_plan_last_kernel.restype = ctypes.c_char_p
    return lib


_lib = _load()


def _check(status, where):
    if status != OK:
        raise CleaveError(status, where)


class Plan:
    """Owns a `cleave_plan*`."""

    def __init__(self, handle):
        self._h = ctypes.c_void_p(handle)
        dims = (ctypes.c_int64 * 3)()
        _check(_lib.cleave_plan_dims(self._h, dims), "cleave_plan_dims")
        self.M, self.N, self.K = int(dims[0]), int(dims[1]), int(dims[2])
        self.num_tasks = int(_lib.cleave_plan_num_tasks(self._h))
        self.num_tiles = int(_lib.cleave_plan_num_tiles(self._h))
        self.partial_elems = int(_lib.cleave_plan_partial_elems(self._h))

    @property
    def tasks(self):
        """Copy of the task list as a structured numpy array."""
        ptr = _lib.cleave_plan_tasks(self._h)
        buf = (ctypes.c_char * (self.num_tasks * TASK_DTYPE.itemsize)).from_address(ptr)
        return np.frombuffer(buf, dtype=TASK_DTYPE).copy()

    def upload(self):
        _check(_lib.cleave_plan_upload(self._h), "cleave_plan_upload")

    @property
    def last_kernel(self):
        return _lib.cleave_plan_last_kernel(self._h).decode()

    def close(self):
        if self._h is not None and self._h.value:
            _lib.cleave_plan_destroy(self._h)
        self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def plan_uniform(M, N, K, tile_m, tile_n, ksplit, gemm_id=0):
    out = ctypes.c_void_p()
    _check(_lib.cleave_plan_uniform(M, N, K, tile_m, tile_n, ksplit, gemm_id, ctypes.byref(out)),
           "cleave_plan_uniform")
    return Plan(out.value)


def plan_explicit(M, N, K, band_h, col_w, ksplit_per_tile, gemm_id=0):
    """band_h: band heights; col_w: one list of widths per band; ksplit_per_tile:
    S per tile, band-major.  The lists are flattened into the C arrays."""
    n_tiles = sum(len(w) for w in col_w)
    if len(col_w) != len(band_h) or len(ksplit_per_tile) != n_tiles:
        raise CleaveError(EINVAL, "plan_explicit (list lengths)")
    bh = np.asarray(band_h, dtype=np.int64)
    nc = np.asarray([len(w) for w in col_w], dtype=np.int32)
    cw = np.asarray([x for w in col_w for x in w], dtype=np.int64)
    ks = np.asarray(ksplit_per_tile, dtype=np.int32)
    out = ctypes.c_void_p()
    _check(_lib.cleave_plan_explicit(M, N, K, len(bh), bh.ctypes.data, nc.ctypes.data,
                                     cw.ctypes.data, ks.ctypes.data, gemm_id, ctypes.byref(out)),
           "cleave_plan_explicit")
    return Plan(out.value)


def _stream_ptr(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if hasattr(stream, "cuda_stream"):
        return ctypes.c_void_p(stream.cuda_stream)
    return ctypes.c_void_p(int(stream))


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("unsupported dtype %s" % t.dtype)


def _matrix(t, what):
    if t.dim() != 2 or t.stride(1) != 1 or not t.is_cuda:
        raise ValueError("%s must be a 2-D device tensor with unit column stride" % what)
    return ctypes.c_void_p(t.data_ptr()), int(t.stride(0))


def execute(plan, A, B, partials, transA=0, transB=0, task_ids=None, stream=None, noalloc=False):
    """cleave_execute (or, with noalloc=True, cleave_execute_noalloc): A, B stored
    device matrices (torch), partials a flat fp32 device tensor of
    plan.partial_elems elements."""
    import torch
    a_ptr, lda = _matrix(A, "A")
    b_ptr, ldb = _matrix(B, "B")
    if A.dtype != B.dtype:
        raise TypeError("A and B must have the same dtype")
    if partials.dtype != torch.float32 or not partials.is_cuda or not partials.is_contiguous() \
            or partials.numel() < plan.partial_elems:
        raise ValueError("partials must be a contiguous fp32 device tensor of partial_elems elements")
    # Stored shapes must hold the logical operands.
    a_rows, a_cols = (plan.K, plan.M) if transA else (plan.M, plan.K)
    b_rows, b_cols = (plan.N, plan.K) if transB else (plan.K, plan.N)
    if tuple(A.shape) != (a_rows, a_cols) or tuple(B.shape) != (b_rows, b_cols):
        raise ValueError("operand shapes %s, %s do not match the plan" % (tuple(A.shape), tuple(B.shape)))
    ids_ptr, n_ids = None, 0
    if task_ids is not None:
        ids = np.ascontiguousarray(task_ids, dtype=np.int64)
        ids_ptr, n_ids = ctypes.c_void_p(ids.ctypes.data), len(ids)
    entry = _lib.cleave_execute_noalloc if noalloc else _lib.cleave_execute
    _check(entry(plan._h, ids_ptr, n_ids, a_ptr, lda, int(transA), b_ptr, ldb,
                 int(transB), _dtype_code(A), ctypes.c_void_p(partials.data_ptr()),
                 _stream_ptr(stream)), "cleave_execute_noalloc" if noalloc else "cleave_execute")


def execute_noalloc(plan, A, B, partials, transA=0, transB=0, task_ids=None, stream=None):
    """cleave_execute_noalloc: as execute, for callers that cannot allocate."""
    execute(plan, A, B, partials, transA, transB, task_ids, stream, noalloc=True)


def reduce(plan, partials, C, stream=None):
    """cleave_reduce: C an M x N device matrix (fp32 or bf16)."""
    c_ptr, ldc = _matrix(C, "C")
    if tuple(C.shape) != (plan.M, plan.N):
        raise ValueError("C must be M x N")
    _check(_lib.cleave_reduce(plan._h, ctypes.c_void_p(partials.data_ptr()), c_ptr, ldc,
                              _dtype_code(C), _stream_ptr(stream)), "cleave_reduce")


def plan_batched(M, N, K, tile_m, tile_n, ksplit, n_batch):
    h = ctypes.c_void_p()
    _check(_lib.cleave_plan_batched(M, N, K, tile_m, tile_n, ksplit, n_batch, ctypes.byref(h)),
           "cleave_plan_batched")
    return Plan(h.value)


def _device_2d(t, what):
    if t.dim() != 2 or t.stride(1) != 1 or not t.is_cuda:
        raise ValueError("%s must be a 2-D device tensor with unit column stride" % what)
    return ctypes.c_void_p(t.data_ptr()), int(t.stride(0))


def execute_batched(plan, A, a_strides, B, b_strides, n_inner, partials, transA=0, transB=0,
                    task_ids=None, stream=None):
    """cleave_execute_batched: A, B are the 2-D device tensors that hold every
    member's operand (leading dimension = their row stride); a_strides /
    b_strides = (outer, inner) element strides between members."""
    import torch
    a_ptr, lda = _device_2d(A, "A")
    b_ptr, ldb = _device_2d(B, "B")
    if A.dtype != B.dtype:
        raise TypeError("A and B must have the same dtype")
    if partials.dtype != torch.float32 or not partials.is_cuda or not partials.is_contiguous() \
            or partials.numel() < plan.partial_elems:
        raise ValueError("partials must be a contiguous fp32 device tensor of partial_elems elements")
    ids_ptr, n_ids = None, 0
    if task_ids is not None:
        ids = np.ascontiguousarray(task_ids, dtype=np.int64)
        ids_ptr, n_ids = ctypes.c_void_p(ids.ctypes.data), len(ids)
    _check(_lib.cleave_execute_batched(
        plan._h, ids_ptr, n_ids, a_ptr, lda, int(transA), int(a_strides[0]), int(a_strides[1]),
        b_ptr, ldb, int(transB), int(b_strides[0]), int(b_strides[1]), int(n_inner),
        _dtype_code(A), ctypes.c_void_p(partials.data_ptr()), _stream_ptr(stream)),
        "cleave_execute_batched")


def execute_assemble(plan, A, B, C, transA=0, transB=0, a_strides=(0, 0), b_strides=(0, 0),
                     c_strides=(0, 0), n_inner=0, task_ids=None, stream=None):
    """cleave_execute_assemble: plans without K-splits write their blocks
    straight into C (fp32 or bf16).  For a batched plan A, B, C are the 2-D
    tensors holding every member and the strides / n_inner say where."""
    a_ptr, lda = _device_2d(A, "A")
    b_ptr, ldb = _device_2d(B, "B")
    c_ptr, ldc = _device_2d(C, "C")
    if A.dtype != B.dtype:
        raise TypeError("A and B must have the same dtype")
    ids_ptr, n_ids = None, 0
    if task_ids is not None:
        ids = np.ascontiguousarray(task_ids, dtype=np.int64)
        ids_ptr, n_ids = ctypes.c_void_p(ids.ctypes.data), len(ids)
    _check(_lib.cleave_execute_assemble(
        plan._h, ids_ptr, n_ids, a_ptr, lda, int(transA), int(a_strides[0]), int(a_strides[1]),
        b_ptr, ldb, int(transB), int(b_strides[0]), int(b_strides[1]), int(n_inner), _dtype_code(A),
        c_ptr, ldc, int(c_strides[0]), int(c_strides[1]), _dtype_code(C), _stream_ptr(stream)),
        "cleave_execute_assemble")


def reduce_batched(plan, partials, C, c_strides, n_inner, stream=None):
    """cleave_reduce_batched: C the 2-D device tensor that holds every member's result."""
    c_ptr, ldc = _device_2d(C, "C")
    _check(_lib.cleave_reduce_batched(plan._h, ctypes.c_void_p(partials.data_ptr()), c_ptr, ldc,
                                      int(c_strides[0]), int(c_strides[1]), int(n_inner),
                                      _dtype_code(C), _stream_ptr(stream)), "cleave_reduce_batched")


def _member_pointers(tensors, what):
    """Host array of the members' device pointers; checks that they share
    dtype and leading dimension."""
    lds = {_device_2d(t, what)[1] for t in tensors}
    if len(lds) != 1 or len({t.dtype for t in tensors}) != 1:
        raise ValueError("%s: members must share dtype and leading dimension" % what)
    arr = (ctypes.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])
    return arr, lds.pop()


def execute_grouped(plan, A_list, B_list, partials, transA=0, transB=0, task_ids=None, stream=None):
    """cleave_execute_grouped: member g of the batched plan multiplies A_list[g]
    by B_list[g] (2-D device tensors; entries may repeat)."""
    import torch
    a_arr, lda = _member_pointers(A_list, "A_list")
    b_arr, ldb = _member_pointers(B_list, "B_list")
    if A_list[0].dtype != B_list[0].dtype:
        raise TypeError("A and B must have the same dtype")
    if len(A_list) != len(B_list):
        raise ValueError("A_list and B_list must have one entry per member")
    if partials.dtype != torch.float32 or not partials.is_cuda or not partials.is_contiguous() \
            or partials.numel() < plan.partial_elems:
        raise ValueError("partials must be a contiguous fp32 device tensor of partial_elems elements")
    ids_ptr, n_ids = None, 0
    if task_ids is not None:
        ids = np.ascontiguousarray(task_ids, dtype=np.int64)
        ids_ptr, n_ids = ctypes.c_void_p(ids.ctypes.data), len(ids)
    _check(_lib.cleave_execute_grouped(plan._h, ids_ptr, n_ids, len(A_list), a_arr, lda, int(transA), b_arr, ldb,
                                       int(transB), _dtype_code(A_list[0]),
                                       ctypes.c_void_p(partials.data_ptr()), _stream_ptr(stream)),
           "cleave_execute_grouped")


def reduce_grouped(plan, partials, C_list, stream=None):
    """cleave_reduce_grouped: member g's result goes to C_list[g]."""
    c_arr, ldc = _member_pointers(C_list, "C_list")
    _check(_lib.cleave_reduce_grouped(plan._h, ctypes.c_void_p(partials.data_ptr()), len(C_list), c_arr, ldc,
                                      _dtype_code(C_list[0]), _stream_ptr(stream)),
           "cleave_reduce_grouped")


def reduce_residual(plan, partials, R, C, stream=None):
    """cleave_reduce_residual: C = sum of partials + R (R may be C)."""
    c_ptr, ldc = _matrix(C, "C")
    r_ptr, ldr = _matrix(R, "R")
    if tuple(C.shape) != (plan.M, plan.N) or tuple(R.shape) != (plan.M, plan.N) or ldr != ldc \
            or R.dtype != C.dtype:
        raise ValueError("R and C must be M x N with the same dtype and leading dimension")
    _check(_lib.cleave_reduce_residual(plan._h, ctypes.c_void_p(partials.data_ptr()), r_ptr, c_ptr,
                                       ldc, _dtype_code(C), _stream_ptr(stream)),
           "cleave_reduce_residual")


def reduce_adam(plan, partials, w, m, v, lr, beta1, beta2, eps, weight_decay, step, w_bf16=None,
                stream=None):
    """cleave_reduce_adam: Adam update of the M x N fp32 weight w (moments m, v)
    with the aggregated partials as gradient; optional bf16 copy of the result."""
    import torch
    w_ptr, ld = _matrix(w, "w")
    ptrs = []
    for t, what, dt in ((m, "m", torch.float32), (v, "v", torch.float32), (w_bf16, "w_bf16", torch.bfloat16)):
        if t is None and what == "w_bf16":
            ptrs.append(None)
            continue
        q, l = _matrix(t, what)
        if t.dtype != dt or tuple(t.shape) != (plan.M, plan.N) or l != ld:
            raise ValueError("%s must be M x N %s with w's leading dimension" % (what, dt))
        ptrs.append(q)
    if w.dtype != torch.float32 or tuple(w.shape) != (plan.M, plan.N):
        raise ValueError("w must be an M x N fp32 device tensor")
    _check(_lib.cleave_reduce_adam(plan._h, ctypes.c_void_p(partials.data_ptr()), w_ptr, ptrs[0],
                                   ptrs[1], ptrs[2], ld, lr, beta1, beta2, eps, weight_decay,
                                   int(step), _stream_ptr(stream)), "cleave_reduce_adam")


def reduce_adam_grouped(plan, partials, w_list, m_list, v_list, lr, beta1, beta2, eps, weight_decay, step,
                        w_bf16_list=None, stream=None):
    """cleave_reduce_adam_grouped: member g of the grouped plan updates w_list[g]
    (moments m_list[g], v_list[g], optional bf16 copy w_bf16_list[g])."""
    w_arr, ld = _member_pointers(w_list, "w_list")
    m_arr, ldm = _member_pointers(m_list, "m_list")
    v_arr, ldv = _member_pointers(v_list, "v_list")
    b_arr = None
    if w_bf16_list is not None:
        b_arr, ldb = _member_pointers(w_bf16_list, "w_bf16_list")
        if ldb != ld or len(w_bf16_list) != len(w_list):
            raise ValueError("w_bf16_list must match w_list")
    if ldm != ld or ldv != ld or not (len(w_list) == len(m_list) == len(v_list)):
        raise ValueError("w, m, v lists must have one entry per member and one leading dimension")
    _check(_lib.cleave_reduce_adam_grouped(plan._h, ctypes.c_void_p(partials.data_ptr()), len(w_list), w_arr,
                                           m_arr, v_arr, b_arr, ld, lr, beta1, beta2, eps, weight_decay,
                                           int(step), _stream_ptr(stream)), "cleave_reduce_adam_grouped")


def verify(plan, A, B, partials, r, s, tol, accept, lhs=None, rhs=None, scale=None,
           transA=0, transB=0, stream=None):
    """cleave_verify: r (M) and s (N) fp32 device vectors, accept an int32 device
    tensor of num_tasks entries; lhs / rhs / scale optional fp64 device tensors
    of num_tasks entries.  Nothing is allocated or computed here."""
    import torch
    a_ptr, lda = _matrix(A, "A")
    b_ptr, ldb = _matrix(B, "B")
    if A.dtype != B.dtype:
        raise TypeError("A and B must have the same dtype")
    a_rows, a_cols = (plan.K, plan.M) if transA else (plan.M, plan.K)
    b_rows, b_cols = (plan.N, plan.K) if transB else (plan.K, plan.N)
    if tuple(A.shape) != (a_rows, a_cols) or tuple(B.shape) != (b_rows, b_cols):
        raise ValueError("operand shapes %s, %s do not match the plan" % (tuple(A.shape), tuple(B.shape)))

    def vec(t, dtype, n, what, optional=False):
        if t is None and optional:
            return None
        if t is None or t.dtype != dtype or not t.is_cuda or not t.is_contiguous() or t.numel() < n:
            raise ValueError("%s must be a contiguous %s device tensor of at least %d entries" % (what, dtype, n))
        return ctypes.c_void_p(t.data_ptr())

    _check(_lib.cleave_verify(
        plan._h, a_ptr, lda, int(transA), b_ptr, ldb, int(transB), _dtype_code(A),
        vec(partials, torch.float32, plan.partial_elems, "partials"),
        vec(r, torch.float32, plan.M, "r"), vec(s, torch.float32, plan.N, "s"), float(tol),
        vec(lhs, torch.float64, plan.num_tasks, "lhs", True),
        vec(rhs, torch.float64, plan.num_tasks, "rhs", True),
        vec(scale, torch.float64, plan.num_tasks, "scale", True),
        vec(accept, torch.int32, plan.num_tasks, "accept"), _stream_ptr(stream)), "cleave_verify")


def _verify_vectors(plan, partials, r, s, accept, lhs, rhs, scale):
    """Pointers of the verify calls' vector arguments for a batched plan (r, s
    hold one probe vector per member)."""
    import torch

    def vec(t, dtype, n, what, optional=False):
        if t is None and optional:
            return None
        if t is None or t.dtype != dtype or not t.is_cuda or not t.is_contiguous() or t.numel() < n:
            raise ValueError("%s must be a contiguous %s device tensor of at least %d entries" % (what, dtype, n))
        return ctypes.c_void_p(t.data_ptr())
    members = r.numel() // plan.M
    return (vec(partials, torch.float32, plan.partial_elems, "partials"),
            vec(r, torch.float32, members * plan.M, "r"), vec(s, torch.float32, members * plan.N, "s"),
            vec(lhs, torch.float64, plan.num_tasks, "lhs", True),
            vec(rhs, torch.float64, plan.num_tasks, "rhs", True),
            vec(scale, torch.float64, plan.num_tasks, "scale", True),
            vec(accept, torch.int32, plan.num_tasks, "accept"))


def schedule_loads(plan, which, grid, balanced=True):
    """cleave_plan_schedule_loads (host only): cost units per workgroup of the
    fast kernel's schedule for list `which` (0 large class, 1 small class, 2
    all-small cut) on `grid` workgroups."""
    loads = np.zeros(int(grid), dtype=np.float64)
    _check(_lib.cleave_plan_schedule_loads(plan._h, int(which), int(grid), int(bool(balanced)),
                                           ctypes.c_void_p(loads.ctypes.data)), "cleave_plan_schedule_loads")
    return loads


def verify_reduce(plan, A, B, partials, r, s, tol, accept, C, lhs=None, rhs=None, scale=None,
                  transA=0, transB=0, stream=None):
    """cleave_verify_reduce: the check of cleave_verify and the aggregation of
    cleave_reduce in one pass over the partial blocks (plain plans)."""
    a_ptr, lda = _matrix(A, "A")
    b_ptr, ldb = _matrix(B, "B")
    c_ptr, ldc = _matrix(C, "C")
    if A.dtype != B.dtype:
        raise TypeError("A and B must have the same dtype")
    if tuple(C.shape) != (plan.M, plan.N):
        raise ValueError("C must be %d x %d" % (plan.M, plan.N))
    pp, rp, sp, lp, hp, cp, ap = _verify_vectors(plan, partials, r, s, accept, lhs, rhs, scale)
    _check(_lib.cleave_verify_reduce(plan._h, a_ptr, lda, int(transA), b_ptr, ldb, int(transB), _dtype_code(A),
                                     pp, rp, sp, float(tol), lp, hp, cp, ap, c_ptr, ldc, _dtype_code(C),
                                     _stream_ptr(stream)), "cleave_verify_reduce")


def verify_batched(plan, A, a_strides, B, b_strides, n_inner, partials, r, s, tol, accept, lhs=None, rhs=None,
                   scale=None, transA=0, transB=0, stream=None):
    """cleave_verify_batched: members addressed as in execute_batched; r is
    [n_batch, M], s is [n_batch, N] (fp32 device tensors)."""
    a_ptr, lda = _device_2d(A, "A")
    b_ptr, ldb = _device_2d(B, "B")
    if A.dtype != B.dtype:
        raise TypeError("A and B must have the same dtype")
    pp, rp, sp, lp, hp, cp, ap = _verify_vectors(plan, partials, r, s, accept, lhs, rhs, scale)
    _check(_lib.cleave_verify_batched(plan._h, a_ptr, lda, int(transA), int(a_strides[0]), int(a_strides[1]),
                                      b_ptr, ldb, int(transB), int(b_strides[0]), int(b_strides[1]), int(n_inner),
                                      _dtype_code(A), pp, rp, sp, float(tol), lp, hp, cp, ap, _stream_ptr(stream)),
           "cleave_verify_batched")


def verify_grouped(plan, A_list, B_list, partials, r, s, tol, accept, lhs=None, rhs=None, scale=None,
                   transA=0, transB=0, stream=None):
    """cleave_verify_grouped: one operand pair per member (as execute_grouped)."""
    a_arr, lda = _member_pointers(A_list, "A_list")
    b_arr, ldb = _member_pointers(B_list, "B_list")
    if A_list[0].dtype != B_list[0].dtype or len(A_list) != len(B_list):
        raise TypeError("A_list and B_list: one entry per member, one dtype")
    pp, rp, sp, lp, hp, cp, ap = _verify_vectors(plan, partials, r, s, accept, lhs, rhs, scale)
    _check(_lib.cleave_verify_grouped(plan._h, len(A_list), a_arr, lda, int(transA), b_arr, ldb, int(transB),
                                      _dtype_code(A_list[0]), pp, rp, sp, float(tol), lp, hp, cp, ap,
                                      _stream_ptr(stream)), "cleave_verify_grouped")


def shard_cost(dev, alpha, beta, n, elem_bytes, alpha_fetch=None, beta_fetch=None):
    """cleave_shard_cost (host only)."""
    c = _lib.cleave_shard_cost(ctypes.byref(dev), alpha, beta,
                               alpha if alpha_fetch is None else alpha_fetch,
                               beta if beta_fetch is None else beta_fetch, n, elem_bytes)
    if c < 0:
        raise CleaveError(EINVAL, "cleave_shard_cost")
    return c


def shard_fits(dev, alpha, beta, n, elem_bytes):
    rc = _lib.cleave_shard_fits(ctypes.byref(dev), alpha, beta, n, elem_bytes)
    if rc < 0:
        raise CleaveError(rc, "cleave_shard_fits")
    return bool(rc)


def assign(m, q, n, elem_bytes, devices, granule, origin=(0, 0), cached=None, mem_used=None):
    """cleave_assign (host only): returns (band_h, col_w, owner, cost) with one
    list of column widths and of owning device indices per band.  With `cached`
    (one (row_lo, row_hi, col_lo, col_hi) per device) and `mem_used`:
    cleave_reassign, the churn re-solve."""
    k = len(devices)
    devs = (Device * max(k, 1))(*devices)
    n_bands = ctypes.c_int32()
    band_h = (ctypes.c_int64 * max(k, 1))()
    n_cols = (ctypes.c_int32 * max(k, 1))()
    col_w = (ctypes.c_int64 * max(k, 1))()
    owner = (ctypes.c_int32 * max(k, 1))()
    cost = ctypes.c_double()
    if cached is None:
        _check(_lib.cleave_assign(m, q, n, elem_bytes, devs, k, granule, ctypes.byref(n_bands), band_h,
                                  n_cols, col_w, owner, ctypes.byref(cost)), "cleave_assign")
    elif cached and len(cached[0]) == 2:
        # general cache sets: one (row_intervals, col_intervals) pair per device -> cleave_reassign_sets
        if mem_used is None or len(cached) != k or len(mem_used) != k:
            raise CleaveError(EINVAL, "assign (cached / mem_used lengths)")
        n_r = (ctypes.c_int32 * max(k, 1))(*[len(c[0]) for c in cached])
        n_c = (ctypes.c_int32 * max(k, 1))(*[len(c[1]) for c in cached])
        r_flat = [int(x) for c in cached for iv in c[0] for x in iv]
        c_flat = [int(x) for c in cached for iv in c[1] for x in iv]
        r_iv = (ctypes.c_int64 * max(len(r_flat), 1))(*r_flat)
        c_iv = (ctypes.c_int64 * max(len(c_flat), 1))(*c_flat)
        used = (ctypes.c_double * max(k, 1))(*[float(x) for x in mem_used])
        _check(_lib.cleave_reassign_sets(m, q, n, elem_bytes, devs, k, granule, int(origin[0]), int(origin[1]),
                                         n_r, r_iv, n_c, c_iv, used, ctypes.byref(n_bands), band_h, n_cols,
                                         col_w, owner, ctypes.byref(cost)), "cleave_reassign_sets")
    else:
        if mem_used is None or len(cached) != k or len(mem_used) != k:
            raise CleaveError(EINVAL, "assign (cached / mem_used lengths)")
        flat = (ctypes.c_int64 * (4 * max(k, 1)))(*[int(x) for c in cached for x in c])
        used = (ctypes.c_double * max(k, 1))(*[float(x) for x in mem_used])
        _check(_lib.cleave_reassign(m, q, n, elem_bytes, devs, k, granule, int(origin[0]), int(origin[1]),
                                    flat, used, ctypes.byref(n_bands), band_h, n_cols, col_w, owner,
                                    ctypes.byref(cost)), "cleave_reassign")
    bands, widths, owners, pos = [], [], [], 0
    for bnd in range(n_bands.value):
        c = n_cols[bnd]
        bands.append(int(band_h[bnd]))
        widths.append([int(x) for x in col_w[pos:pos + c]])
        owners.append([int(x) for x in owner[pos:pos + c]])
        pos += c
    return bands, widths, owners, cost.value


def version():
    return int(_lib.cleave_version())
