"""MI355X-native LOOKAT: attention decode over a product-quantised key cache.

The work is done by hand-written HIP kernels for gfx950 behind the C ABI declared in
``include/lookat.h`` (``liblookat.so``).  This package is the thin Python binding:
argument marshalling from torch tensors (device memory and streams) to that ABI.
There is no CPU fallback: without the built library every call raises.
"""
from .binding import (  # noqa: F401
    LookatError,
    attend_decode,
    attend_decode_auto_splits,
    attend_decode_launch_shape,
    attend_decode_gqa_workspace_bytes,
    attend_decode_workspace_bytes,
    build_lut,
    encode_keys,
    last_error,
    lib_path,
    load_library,
    lookat_attend_decode,
    lookat_attend_decode_gqa,
    lookat_attend_decode_noalloc,
    lookat_build_lut,
    lookat_decode_step,
    lookat_decode_step_split,
    lookat_decode_step_gqa,
    decode_step_split_workspace_bytes,
    decode_step_entries_per_workgroup,
    lookat_encode_keys,
    lookat_kmeans,
    lookat_kmeans_step,
    lookat_probe_attend_decode_ticket,
    lookat_probe_score_prefill_lookup,
    lookat_probe_decode_step_entries,
    lookat_probe_empty_launch,
    lookat_probe_stream_read,
    lookat_probe_stream_read_shaped,
    probe_attend_decode_ticket_workspace_bytes,
    lookat_probe_stream_write,
    lookat_score_prefill,
    version,
)

__all__ = [
    "LookatError", "attend_decode", "attend_decode_auto_splits", "attend_decode_launch_shape", "attend_decode_gqa_workspace_bytes", "attend_decode_workspace_bytes",
    "build_lut", "encode_keys", "last_error", "lib_path", "load_library", "version",
    "lookat_attend_decode", "lookat_attend_decode_gqa", "lookat_attend_decode_noalloc", "lookat_build_lut", "lookat_decode_step", "lookat_decode_step_split", "lookat_decode_step_gqa", "decode_step_split_workspace_bytes", "decode_step_entries_per_workgroup", "lookat_encode_keys", "lookat_kmeans", "lookat_kmeans_step",
    "lookat_probe_stream_read", "lookat_probe_stream_read_shaped", "lookat_probe_empty_launch", "lookat_probe_attend_decode_ticket", "lookat_probe_score_prefill_lookup", "lookat_probe_decode_step_entries", "probe_attend_decode_ticket_workspace_bytes", "lookat_probe_stream_write", "lookat_score_prefill",
]
