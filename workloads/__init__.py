"""Seeded synthetic inputs for the batched variant-selection path.

This package only draws random tables and query streams.  It contains none of
the selection method's arithmetic, so both the CPU oracle's tests and the GPU
path's tests may use it without sharing any code of the method itself.
"""
from .configs import (  # noqa: F401
    CONFIG_NAMES,
    VariantTable,
    QueryBatch,
    LoadUpdate,
    config_spec,
    make_table,
    make_queries,
    make_load_update,
    make_degrading_load_update,
    make_cliff_table,
    base_seed,
    VariantStates,
    StateUpdate,
    make_states,
    make_state_update,
    WorkerTables,
    WorkerUpdate,
    make_workers,
    make_worker_update,
    make_instance_states,
    make_instance_state_update,
    ScalingProfile,
    ScaleRequests,
    make_scaling,
    make_scale_down_requests,
    make_scale_requests,
)
