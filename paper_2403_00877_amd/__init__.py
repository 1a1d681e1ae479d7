"""MI355X-native tower hot path of Disaggregated Multi-Tower (arXiv 2403.00877).

`binding` mirrors the C ABI of libdmt.so (include/dmt.h) one to one.
"""
from .binding import (  # noqa: F401
    DmtError, dmt_plan, dmt_plan_create, dmt_plan_layout, dmt_plan_bind,
    dmt_tower_lookup_fwd, make_tm_params, dmt_tm_workspace_bytes, dmt_tower_module_fwd,
    make_tm_grads, dmt_tm_bwd_workspace_bytes, dmt_tower_module_bwd,
    dmt_tm_kept_bytes, dmt_tower_module_fwd_keep,
    dmt_bwd_workspace_bytes, dmt_tower_lookup_bwd_update, dmt_last_device_error,
    status_str, library_path, dmt_kernel_name, dmt_profile_enable, dmt_profile_read,
    DMT_K_COUNT, EXPORTS, dmt_calibration_copy, dmt_calibration_gather,
    dmt_tp_workspace_bytes, dmt_tp_interaction, dmt_tp_embed, dmt_tp_kmeans,
    dmt_sptt_peer_order, dmt_sptt_peer_permute, dmt_sptt_shuffle, dmt_plan_set_row_shards,
    dmt_bwd_noalloc_scratch_bytes, dmt_tower_lookup_bwd_update_noalloc, dmt_sptt_peer_permute_ids)
