"""MI355X-native forest verification for dynamic-width speculative beam decoding.

Thin Python binding over libdsbd.so (hand-written HIP for gfx950).  PyTorch is used only for
device memory and streams; every step of the path runs in the library's kernels.  Importing
this package fails loudly if the library has not been built (python -m paper_2409_16560_amd.build).
"""
from .binding import (  # noqa: F401
    DsbdError, Forest, PrefixKV, VerifyResult, NextBeams, KVDst, lib_path, load_library,
    dsbd_forest_attention, dsbd_verify_forest, dsbd_verify_forest_select, dsbd_select_beams, dsbd_commit_kv, dsbd_draft_layer, dsbd_build_forest,
    dsbd_version,
    dsbd_forest_attention_workspace_bytes, dsbd_verify_forest_workspace_bytes,
    dsbd_timing_enable, dsbd_timing_collect, dsbd_reload_knobs, dsbd_stream_read_probe, dsbd_init, dsbd_verify_forest_static, dsbd_verify_forest_static_capacity, DSBD_KERNEL_ATTENTION, DSBD_KERNEL_VOCAB_STATS, DSBD_KERNEL_VERIFY_LAYERS, DSBD_KERNEL_KV_COMMIT,
    DSBD_NOT_REACHED, DSBD_ACCEPTED, DSBD_REJECTED, DSBD_PRUNED, DSBD_ROOT,
    DSBD_FAULT_TOPOLOGY, DSBD_FAULT_TOKEN, DSBD_FAULT_NONFINITE, DSBD_FAULT_ZERO_RESIDUAL,
    DSBD_FAULT_BOUNDS, DSBD_FAULT_SYNC_TIMEOUT,
)
