"""CPU oracle for the sharded weight-update path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, numpy implementation of what the HIP library computes, written
from the paper's description (Sections 2.2, 4.1, 4.2, 5.1, 5.2) and from the published
definitions of Adam, momentum SGD, LAMB, LARS and Adafactor.  It shares no code with the HIP
path and must never be imported by it: only tests, the smoke check and the
benchmark's cpu_baseline leg may use it.

Precision: optimizer state is stored in float32 (the paper keeps the weight
update in float32, Section 4.2); the arithmetic of one step is carried out in
float64 on those float32 values and rounded to float32 once, when the step's
results are stored.  Norm sums are float64.

Every function here is pinned by tests/test_oracle_*.py against the paper's
worked shape examples, closed forms, brute force on tiny inputs and library
routines; no function is "parity unpinned".
"""
from .plan import Plan, make_plan, make_row_plan  # noqa: F401
from .formatting import shard_format, unshard_format, f32_to_bf16_bits, bf16_bits_to_f32  # noqa: F401
from .optim import (  # noqa: F401
    adam_step, momentum_step, lamb_unsharded_step, lamb_shard_partials, lamb_shard_apply,
    lars_unsharded_step, lars_shard_partials, lars_shard_apply,
    rowcol_sumsq_unsharded, rowcol_sumsq_shard,
    VAR_NO_DECAY, VAR_NO_ADAPT,
)
from .adafactor import (  # noqa: F401
    adafactor_schedule, adafactor_second_moment, adafactor_unsharded_step,
    adafactor_shard_partials, adafactor_shard_moments, adafactor_shard_apply,
)
from .topology import (  # noqa: F401
    partial_sharding, two_phase_shard_id, concat_partition, peak_memory, plan_peak_bytes,
)
