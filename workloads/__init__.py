"""Seeded synthetic workloads shaped like the paper's Infinity-2B / 8B runs.

This package serves both the HIP path and the CPU oracle with *inputs only*:
the scale schedules, the per-(layer, scale) budgets and roles, and the seeded
Q/K/V tensors.  It contains none of the method's arithmetic (no softmax, no
scoring, no selection, no attention), imports neither the HIP binding nor the
oracle, and is imported by both test sides so that they see the same bits.
"""
from .configs import (  # noqa: F401
    CONFIGS,
    WorkloadConfig,
    StepPlan,
    get_config,
    c_full,
    layer_roles,
    budget_table,
    window_indices,
    step_plans,
    dst_capacity,
    final_scale_budgets,
    stream_key,
    FINAL_SCALE_BUDGET_FRACS,
)
from .generator import (  # noqa: F401
    normal_tensor,
    student_t_tensor,
    sign_tensor,
    StepInputs,
    FinalScaleCase,
    make_prefix,
    make_step_inputs,
    make_final_scale_case,
    AsiCase,
    asi_sample_rows,
    assemble_asi_case,
    make_asi_case,
)
