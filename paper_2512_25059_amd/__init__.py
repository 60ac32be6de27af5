"""MI355X-native hot path of a resilient ring all-reduce (R2CCL): thin Python binding.

Every step runs in the HIP kernels of ``libr2ccl.so``; this package only marshals
arguments (torch tensors -> device pointers, the current torch stream -> hipStream_t).
There is no CPU fallback: without the built library, calls raise.
"""
from .binding import (  # noqa: F401
    BF16,
    F32,
    OP_COPY,
    OP_SUM,
    PHASE_AG,
    PHASE_AR,
    PHASE_RS,
    R2Error,
    ReduceCopyCall,
    SCHED_AUTO,
    SCHED_FUSED,
    SCHED_STEPS,
    SimCall,
    SimDesc,
    library_path,
    r2_bridge_rerank,
    load_library,
    r2_partition,
    r2_partition_device,
    r2_reduce_copy,
    r2_rollback_plan_device,
    r2_ring_allreduce_sim,
    r2_sim_fused_steps,
    r2_sim_num_passes,
    r2_sim_num_steps,
    r2_sim_num_transmissions,
    r2_sim_prepare,
    r2_sim_resolve_schedule,
    r2_sim_stage_capacity,
    r2_sim_stage_offset,
    r2_sim_step,
    r2_sim_workspace_bytes,
    r2_strerror,
)
