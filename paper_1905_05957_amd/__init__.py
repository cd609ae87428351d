"""MI355X-native DoubleSqueeze step: hand-written HIP kernels behind a C-ABI (libds_hip.so).

This package is the thin Python binding: argument marshalling only.  Every step of the path
(error compensation, compression, aggregation, update) runs in the library's kernels.
PyTorch provides device memory and streams, nothing else.
"""
from .binding import (  # noqa: F401
    COMP_CLIP, COMP_IDENTITY, COMP_RSPARSE, COMP_SIGN, COMP_TERNARY, COMP_TOPK, COMP_QSGD, FLAG_DEFERRED_ERROR, FLAG_NO_ERROR_FEEDBACK, FLAG_SERVER_IDENTITY, FLAG_SIGN_RMS, FLAG_TOPK_MULTI_LAUNCH, SCALE_WHOLE, SCALE_SEGMENTS, SCALE_CHUNK,
    Context, DsError, Payload, ds_apply_update, ds_create, ds_decompress, ds_destroy, ds_materialize_error,
    ds_payload_sizes, ds_probe_copy, ds_server_aggregate_compress, ds_server_aggregate_compress_update, ds_worker_compress, ds_worker_compress_sign_noalloc, library_path, load_library,
)
