"""The host-side rows (cost model, shard assignment, churn re-solve, task
plans) once more under the `gpu` marker: they need no GPU, but the GPU job is
the record of what ran against the built library on the target machine."""
import pytest

import test_plan_parity
import test_scheduler_independent as ind
import test_scheduler_parity as par

pytestmark = pytest.mark.gpu


def test_cost_model_and_assignment_parity_on_the_gpu_box():
    par.test_shard_cost_and_fit_are_bit_equal()
    for case in par.CASES[2:]:
        par.test_assignment_is_identical_to_the_oracles(*case)
    par.test_churn_resolve_is_identical_to_the_oracles(2048, 1536, 1024, 12, 64, 77)
    par.test_assignment_rejects_bad_input_and_infeasible_memory()


def test_assignment_against_the_exact_guillotine_optimum_on_the_gpu_box():
    ind.test_bottleneck_assignment_by_hand()
    for seed in range(10):
        ind.test_library_against_the_exact_guillotine_optimum(seed)
    ind.test_library_layout_is_valid_and_above_the_lower_bounds_at_scale(4096, 11008, 4096, 100, 64, 2)


def test_library_exports_on_the_gpu_box():
    test_plan_parity.test_library_exports_every_declared_symbol()
