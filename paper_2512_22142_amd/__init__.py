"""MI355X-native sub-GEMM task executor and partial reducer (Cleave's hot path).

    plan_uniform / plan_explicit  -> Plan (task list in canonical order)
    execute(plan, A, B, partials) -> fp32 partial blocks, one per task
    reduce(plan, partials, C)     -> C = fixed-order sum of each tile's partials
    verify(plan, A, B, partials, r, s, tol, accept) -> per-task random-projection check

All compute happens in libcleave.so (hand-written HIP for gfx950, C ABI in
include/cleave.h); build it with `python -m paper_2512_22142_amd.build`.
"""
from .binding import (  # noqa: F401
    BF16, F32, CleaveError, Device, Plan, assign, shard_cost, shard_fits, TASK_DTYPE, EXPORTS, LIB_PATH,
    execute, execute_assemble, execute_batched, plan_batched, plan_explicit, plan_uniform, reduce, reduce_adam, reduce_batched,
    reduce_residual, verify, version,
)
