"""MI355X-native ChunkKV prefill-time KV-cache compression (arXiv 2502.00299).

The package is a thin binding over libchunkkv.so (hand-written HIP for gfx950 behind a C ABI, see
include/chunkkv.h).  PyTorch only provides device memory and streams.
"""
from .binding import (  # noqa: F401
    BF16,
    F16,
    F32,
    FLAG_TWO_PASS,
    FLAG_WHOLE_CHUNKS,
    LIB_PATH,
    SYMBOLS,
    ChunkKVError,
    Problem,
    chunkkv_chunk_topk,
    chunkkv_compact,
    chunkkv_compress_layer,
    chunkkv_quality_metrics,
    chunkkv_quality_workspace_bytes,
    chunkkv_compress_stack_hybrid,
    chunkkv_workspace_bytes_hybrid,
    chunkkv_compress_stack,
    chunkkv_compress_stack_lse,
    chunkkv_decode_attention,
    chunkkv_decode_attention_static,
    chunkkv_decode_workspace_bytes,
    chunkkv_jaccard,
    chunkkv_score,
    chunkkv_score_lse,
    chunkkv_status_string,
    chunkkv_timing_begin,
    chunkkv_timing_end,
    TIMING_KINDS,
    chunkkv_workspace_bytes,
    load_library,
)
