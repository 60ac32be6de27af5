"""CPU oracle for the resilient ring all-reduce hot path.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg.  The product package never imports it and it
never imports the product package.

``r2_oracle`` (plain C behind ctypes) holds the partition, the fused reduce-copy, the ring step by
step and the ring's result by definition; the other modules compose those in Python:
``split`` and ``recursive`` (the failure-aware all-reduce schedules and their planners),
``rerank`` (bridge re-ranking), ``sendrecv`` and ``collectives`` (the other collectives under
R2CCL-Balance), ``rails`` (rings whose servers each have a channel state of their own), ``inflight`` (the ring when a
channel fails while a transmission is in flight).
"""
from .r2_oracle import (  # noqa: F401
    BF16,
    F32,
    OP_COPY,
    OP_SUM,
    OP_SUM_FORWARD,
    PHASE_AG,
    PHASE_AR,
    PHASE_RS,
    NoHealthyChannel,
    OracleError,
    bf16_to_f32,
    build,
    expected,
    f32_to_bf16,
    num_steps,
    num_transmissions,
    partition,
    reduce_copy,
    ring_sim,
    rollback_plan,
    set_threads,
    threads,
)
