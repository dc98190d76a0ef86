"""MI355X-native pack / restore of KV caches as video-frame planes (KVCodec hot path).

Thin binding over libkvc.so (see include/kvc.h): argument marshalling only,
every step runs in the HIP kernels.  There is no CPU fallback: importing works
anywhere, calling needs the built library and a gfx950 GPU.
"""
from .kvc import (  # noqa: F401
    KVC_BF16, KVC_F16, KVC_ORDER_CHUNK, KVC_ORDER_LAYER, KVC_Q_PER_CHANNEL, KVC_Q_PER_TOKEN, KvcError, Layout,
    admission_min_buffered, admission_ok, blob_meta_offset, chunk_sizes, est_bandwidth, frame_offset, frame_size,
    layout_set_resolution, meta_staging_size, pack_plan, build_id, select_resolution, kvc_fetch_pipeline, kvc_fetch_pipeline_frames, kvc_pack, kvc_restore, kvc_restore_paged,
    kvc_restore_paged_frame, kvc_restore_paged_frames, layout_validate, lib_path, load, status_str, N_RESIDUALS, residual_histograms_size,
    kvc_residual_histograms, proxy_cost_bits, tile_candidates, kvc_probe_expand, PROBE_ONE_XCD_PER_PIECE, PROBE_LINE_READS,
)
