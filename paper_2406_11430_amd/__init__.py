"""L2-norm KV-cache compression and decode attention for AMD MI355X (gfx950).

Python face of libl2kv.so (see include/l2kv.h): the functions below have the
names of the C entry points and only marshal arguments.  ``synth`` holds the
seeded input generators and none of the method's arithmetic.
"""
from .binding import (  # noqa: F401
    L2KV_BF16, L2KV_F32, L2KV_KEEP_HIGHEST, L2KV_KEEP_LOWEST, L2KVError, LIB_PATH, lib,
    l2kv_compact, l2kv_decode_attn, l2kv_decode_attn_splits, l2kv_decode_max_splits,
    l2kv_decode_workspace_bytes, l2kv_keep_count, l2kv_norms, l2kv_select, l2kv_select_k,
    l2kv_select_workspace_bytes, l2kv_version, l2kv_select_ragged, l2kv_compact_ragged,
    l2kv_stream_append, l2kv_stream_evict, l2kv_decode_attn_ragged, l2kv_decode_ragged_workspace_bytes, l2kv_random_keys, l2kv_decode_workspace_init,
    l2kv_norm_ranks, l2kv_norm_ranks_workspace_bytes, l2kv_alr, l2kv_alr_workspace_bytes,
    l2kv_length_order, l2kv_decode_attn_static, l2kv_device_info, l2kv_compress, l2kv_decode_attn_out, l2kv_read_probe,
)
