"""MI355X (gfx950) streaming attention path of VideoScan: thin Python binding over
libvideoscan.so.  All arithmetic runs in the HIP kernels behind the C ABI declared in
include/videoscan.h; this package only marshals torch device tensors into pointers."""
from .binding import (  # noqa: F401
    VSError,
    VS_BF16,
    VS_F32,
    Cache,
    Shape,
    carrier_compact_append,
    carrier_compact_append_batched,
    carrier_mean_pool,
    current_stream_handle,
    decode_attn,
    frame_prefill_attn,
    frame_prefill_compact,
    lib,
    set_tuning,
    TUNE_PREFILL_SPLITS,
    TUNE_PREFILL_KV_GROUPS,
    TUNE_DECODE_CHUNK_ROWS,
    TUNE_SKIP_MERGE,
    TUNE_PREFILL_MERGE,
    lib_path,
    status_string,
    workspace_bytes,
    workspace_init,
    make_workspace,
)
