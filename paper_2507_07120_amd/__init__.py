"""MI355X-native hot path of Helix Parallelism's attention phase: per-shard decode attention with a
log-sum-exp per head, and the LSE rescale-and-sum combine (Sec. 2.1.1, Fig. 4 top).

The work is done by the HIP library ``libhelix_attn.so`` (C ABI in ``include/helix_attn.h``); this
package only marshals arguments.  There is no CPU fallback: without the built library every call
raises.
"""
from .binding import (  # noqa: F401
    HelixError,
    HopbBuffers,
    KV_BF16,
    KV_FP8_E4M3,
    KV_MXFP4,
    KVShard,
    Problem,
    helix_attn_combine,
    helix_attn_decode,
    helix_attn_decode_hopb,
    helix_attn_decode_kvp,
    helix_attn_decode_static,
    helix_attn_hopb_workspace_bytes,
    helix_attn_partial,
    helix_attn_plan,
    helix_attn_workspace_bytes,
    helix_hopb_span,
    helix_kv_append,
    helix_kv_append_mxfp4,
    helix_kv_append_owner,
    helix_kv_read_seconds,
    helix_probe_mfma_lds,
    helix_probe_stream_read,
    helix_shard_layout,
    helix_status_string,
    helix_weight_read_seconds,
    library_path,
    load_library,
)
