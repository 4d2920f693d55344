"""CPU float64 oracle of the Natural GaLore optimizer step.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this package:
only the test-suite, the smoke check and the benchmark's CPU-baseline leg do.
It shares no code with the HIP library and never imports it.
"""
from .natural_galore import (  # noqa: F401
    HParams,
    OracleState,
    adam_direction,
    adam_moments,
    back_project_update,
    back_project_update_right,
    carry_history,
    fisher_history_matrix,
    init_state,
    natural_gradient_transform,
    project,
    project_right,
    push_history,
    refresh_projector,
    round_to_bf16,
    step,
    top_r_left_singular_vectors,
    top_r_right_singular_vectors,
)
