"""MI355X-native sub-GEMM task executor and partial reducer (Cleave's hot path).

    plan_uniform / plan_explicit  -> Plan (task list in canonical order)
    execute(plan, A, B, partials) -> fp32 partial blocks, one per task
    reduce(plan, partials, C)     -> C = fixed-order sum of each tile's partials
    verify(plan, A, B, partials, r, s, tol, accept) -> per-task random-projection check

All compute happens in libcleave.so (hand-written HIP for gfx950, C ABI in
include/cleave.h); build it with `python -m paper_2512_22142_amd.build`.
"""
# The binding (and with it libcleave.so) is loaded on first use of any of these
# names, so that `paper_2512_22142_amd.build` can be imported in a tree where
# the library has not been built yet.  There is no fallback: if the library is
# missing, the first use raises ImportError.
_BINDING_NAMES = (
    "BF16",
    "F32",
    "OK",
    "EINVAL",
    "ENOMEM",
    "EHIP",
    "ELIMIT",
    "CleaveError",
    "Device",
    "Plan",
    "assign",
    "shard_cost",
    "shard_fits",
    "TASK_DTYPE",
    "EXPORTS",
    "LIB_PATH",
    "execute",
    "execute_assemble",
    "execute_batched",
    "execute_grouped",
    "execute_noalloc",
    "plan_batched",
    "plan_explicit",
    "plan_uniform",
    "reduce",
    "reduce_adam",
    "reduce_adam_grouped",
    "reduce_batched",
    "reduce_grouped",
    "reduce_residual",
    "schedule_loads",
    "verify",
    "verify_batched",
    "verify_reduce",
    "verify_grouped",
    "version",
)


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError("module %r has no attribute %r" % (__name__, name))


def __dir__():
    return sorted(list(globals()) + list(_BINDING_NAMES))
