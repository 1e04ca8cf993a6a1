"""MI355X-native DS-Sync hot path: worker division, fused local-SGD + in-group
parameter average, consensus deviation.  The work is done by hand-written HIP
kernels in ``libdssync.so`` (C ABI: ``include/dssync.h``); this package only
marshals arguments."""
from .binding import (ds_group_sync_opt, ds_group_sync_ragged_opt, ds_local_opt, local_opt, DS_BF16, DS_F32, DS_MAX_W, DsError, ds_consensus, ds_consensus_grouped, ds_consensus_static, ds_consensus_workspace_bytes,
                      ds_group_sync, ds_group_sync_tiled, ds_consensus_tiled, ds_consensus_grouped_tiled, ds_group_sync_consensus_tiled, ds_tiled_elements, ds_group_sync_consensus, ds_group_sync_consensus_workspace_bytes, ds_group_sync_ragged, ds_partition, ds_pattern, ds_pattern_check, ds_pattern_period,
                      ds_padded_ld, DS_MAX_COLUMNS, ds_ragged_plan,
                      ds_ragged_plan_bytes, pack_segments, status_string)

from .layerwise import LayerwiseSync

__all__ = ["LayerwiseSync", "ds_group_sync_opt", "ds_group_sync_ragged_opt", "ds_local_opt", "local_opt", "DS_BF16", "DS_F32", "DS_MAX_W", "DsError", "ds_consensus", "ds_consensus_grouped", "ds_consensus_static", "ds_consensus_workspace_bytes",
           "ds_group_sync", "ds_group_sync_tiled", "ds_consensus_tiled", "ds_consensus_grouped_tiled", "ds_group_sync_consensus_tiled", "ds_tiled_elements", "ds_group_sync_consensus", "ds_group_sync_consensus_workspace_bytes", "ds_group_sync_ragged", "ds_partition", "ds_pattern", "ds_pattern_check", "ds_pattern_period",
           "ds_padded_ld", "DS_MAX_COLUMNS", "ds_ragged_plan", "ds_ragged_plan_bytes",
           "pack_segments", "status_string"]
