"""MI355X-native parallel-drafting attention of the P-EAGLE drafter (training hot path).

Thin ctypes binding over ``libpeagle_attn.so`` (C ABI in ``include/peagle.h``).  PyTorch is
used only for device buffers and streams; every step of the path runs in the HIP kernels.
"""
from .binding import (  # noqa: F401
    ASSIGN_ALGORITHM1,
    ASSIGN_BY_ANCHOR,
    DecodeShape,
    PeagleError,
    Shape,
    TileMap,
    lib_path,
    load_library,
    peagle_attn_bwd,
    peagle_attn_fwd,
    peagle_attn_step_partitioned,
    peagle_attn_step_partitioned_rope,
    peagle_attn_step_profiled,
    peagle_attn_step_rope_profiled,
    peagle_attn_step_rope_shared,
    peagle_rope_shared_workspace_bytes,
    peagle_rope_position_ids,
    peagle_rope_positions,
    peagle_rope_rotate,
    peagle_rope_table,
    peagle_rope_workspace_bytes,
    peagle_build_tilemap_packed,
    peagle_build_tilemap_sampled,
    peagle_measure_mfma_ceiling,
    peagle_build_tilemap,
    peagle_device_info,
    peagle_draft_decode,
    peagle_draft_decode_splits,
    peagle_draft_decode_static,
    peagle_draft_decode_workspace_bytes,
    peagle_strerror,
    peagle_workspace_bytes,
)
