"""MI355X-native sharded weight update: Python binding of libshardupdate.so.

The library itself (HIP kernels + C ABI) lives in csrc/ and include/shardupdate.h; this package
only marshals arguments.  Importing it does not load the library; the first call does.
"""
from ._lib import ShardError, lib  # noqa: F401
from .api import (  # noqa: F401
    FullTensors, KERNEL_IDS, SHARD_BF16, SHARD_F32, SHARD_VAR_NO_ADAPT, SHARD_VAR_NO_DECAY, Plan,
    gathered_empty, shard_format, shard_format_all, shard_plan, shard_plan_rows, shard_plan_rowcol_layout, shard_reduce_sq_rows_cols, shard_plan_bind, shard_profile_enable, shard_profile_read, shard_profile_reset, shard_profile_plain_copy, shard_profile_adam_shape,
    shard_plan_set_copy_walk, shard_plan_copy_walk, shard_plan_tune_copy_walk, COPY_WALKS, shard_plan_release_captured_tables,
    shard_update_adam, shard_update_lars, shard_update_lars_apply, shard_update_lars_partials, shard_update_lamb, shard_update_lamb_apply, shard_update_lamb_partials, shard_update_lamb_full_grads, shard_update_lamb_noalloc, shard_update_lamb_partials_full_grads, shard_update_adam_full_grads,
    shard_update_momentum_full_grads, shard_update_lars_full_grads, shard_update_lars_partials_full_grads,
    shard_update_lars_apply_full_grads,
    shard_update_momentum, unshard_format,
    shard_update_adafactor, shard_update_adafactor_partials, shard_update_adafactor_moments, shard_update_adafactor_apply,
    shard_partial_sharding, shard_two_phase_shard_id, shard_concat_partition, shard_peak_memory, shard_plan_peak_bytes,
)
from .build import build_library  # noqa: F401
