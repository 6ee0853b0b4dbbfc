"""One GPU's share of StarTrail / ring attention for gfx950 (MI355X).

The work is done by hand-written HIP kernels behind a C ABI (``include/startrail.h``,
``libstartrail.so``); this package only marshals arguments.  PyTorch tensors are used as
device-memory handles and for the current HIP stream.  There is no CPU fallback: importing
the bindings without the built library raises.
"""
from .api import (  # noqa: F401
    ST_BF16, ST_F32, ST_KV_ASSIGN, ST_RING_FUSED, ST_RING_STEPWISE, StarTrailError,
    st_attn_block_bwd, st_attn_block_bwd_workspace_bytes, st_attn_block_fwd, st_attn_combine, st_attn_delta, st_attn_merge, st_cast_from_f32,
    st_last_error, st_ring_bwd, st_ring_bwd_last, st_ring_bwd_noalloc, st_ring_bwd_noalloc_max_bytes, st_ring_fwd, st_ring_workspace_bytes, st_status_str,
    st_version, st_visit_order, st_team_visit_order, st_schedule_report, library_path, st_profile_begin, st_profile_end, st_device_facts, st_mfma_probe, st_mfma_probe_mixes, st_mfma_probe_mix_name,
)
