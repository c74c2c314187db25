"""MI355X (gfx950) hierarchical recursive-doubling all-reduce (Algorithm 1 of the paper),
emulated over P resident buffers on one GPU.  All work happens in librar.so (HIP kernels
behind the C ABI declared in include/rar.h); this package only marshals arguments."""
from .binding import (  # noqa: F401
    RAR_BF16, RAR_F32, RAR_MODE_AUTO, RAR_MODE_FUSED, RAR_MODE_FUSED_PACKED, RAR_MODE_STEPWISE, RarError, AllReduce, lib,
    rar_allreduce, rar_allreduce_chain, rar_allreduce_static, rar_plan_static_bytes, RAR_STATIC_SCRATCH_BYTES, rar_autotune, rar_barrier_only, rar_copy_probe, rar_launch_floor, rar_plan, rar_plan_chunk,
    rar_plan_effective_mode, rar_plan_fold_partner, rar_plan_free, rar_plan_get_mode, rar_plan_get_tuning, rar_plan_nodes, rar_plan_peer,
    rar_plan_ranks, rar_plan_scratch_bytes, rar_plan_scratch_layout, rar_plan_set_concurrency, rar_plan_set_mode, rar_plan_set_scratch,
    rar_plan_set_tuning, rar_plan_set_wait_limit_us, rar_plan_status, rar_plan_steps,
    rar_read_probe, rar_step_combine, rar_strerror, rar_version)
