"""CPU oracle for the ragged, batch-size-weighted SGD step (test infrastructure).

Plain, slow, fp64 / exact-integer reference of what the GPU library computes,
written from the paper's equations.  It shares no code with the HIP path and is
only ever imported by the tests, the smoke check and the benchmark's CPU
baseline leg; the product path never calls it.

Pinned by tests/test_oracle_*.py against values the paper fixes (the
heterogeneity-level table fed through the variable-batching equation), closed
forms, finite differences, brute-force loops and an independent autograd
library.  Parity unpinned: the free-running 200-step bf16 trajectory (only
single-step, teacher-forced comparisons are pinned).
"""
from .controller import (
    InfeasibleError,
    apportion,
    controller_run,
    global_batch_rule,
    offsets,
    proportional_update,
)
from .step import forward_backward, sgd_step, StepResult

__all__ = [
    "InfeasibleError", "apportion", "controller_run", "global_batch_rule", "offsets",
    "proportional_update", "forward_backward", "sgd_step", "StepResult",
]
