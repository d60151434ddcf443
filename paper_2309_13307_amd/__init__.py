"""MI355X-native hot path of CORE (Common Random Reconstruction, arXiv 2309.13307).

The product is the C-ABI library ``libcore_hip.so`` (see ``include/core.h``); this package is its
thin Python binding plus the seeded synthetic-input generators used by tests and the benchmark.
"""
from .binding import (  # noqa: F401
    CoreError, alloc_workspace, core_compress, core_compress_batched, core_debug_philox,
    core_debug_xi, core_reconstruct, core_round, core_workspace_bytes, load_library, strerror,
    alloc_xi, core_compress_batched_store_xi, core_reconstruct_from_xi, core_round_materialized,
    core_xi_bytes, core_reconstruct_update, core_round_update,
    core_projection_sqnorms, core_privacy_loss,
    core_nonconvex_step, core_step_size_option2, core_reconstruct_trial, core_round_trial,
    core_accept_trial, core_debug_plan, core_round_update_r, core_advance_round, core_round_trial_r,
    core_reconstruct_update_batched, core_build_id, core_debug_philox_layout, core_debug_set_projection,
    core_round_static,
)
