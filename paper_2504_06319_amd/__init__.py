"""Paged-KV decode attention with asynchronous KV-block prefetch for AMD MI355X (gfx950).

The compute lives in hand-written HIP kernels behind a C ABI (``csrc/``, declared in
``include/kvprefetch.h``); ``binding`` marshals torch tensors into it.
"""
from .binding import (  # noqa: F401
    KVError,
    KV_MAX_PREFETCH_DISTANCE,
    kv_decode_attn,
    kv_decode_attn_kv8,
    kv_decode_attn_noalloc,
    KV_NOALLOC_SCRATCH_BYTES,
    kv_decode_get_waves_per_cu_kv8,
    kv_decode_layerstack,
    kv_decode_workspace_bytes,
    kv_layerstack_workspace_bytes,
    kv_decode_set_worker_trace,
    kv_decode_set_xcd_skew,
    kv_decode_set_l2_touch,
    kv_decode_set_variant,
    kv_decode_get_waves_per_cu_for,
    KV_VARIANT_ONE_PASS,
    KV_VARIANT_TWO_PHASE,
    kv_decode_fetch_probe,
    kv_decode_set_waves_per_cu,
    kv_decode_get_waves_per_cu,
    kv_block_bytes,
    kv_worker_range,
    kv_worker_of_tile,
    kv_profile_enable,
    kv_profile_read,
    kv_profile_read_each,
    kv_iter_working_set_bytes,
    kv_version,
    kv_last_error,
    load_library,
    pack_weights,
    library_path,
)
