"""MI355X-native turn-resumption kernels (K,V pack / unpack, prefix-cached prefill attention).

A thin binding over the C-ABI library ``libsymph.so`` (see ``include/symph.h``): argument marshalling only,
every step of the path runs in the HIP kernels.  Importing this package does not touch the GPU; the library
is loaded on first use and a missing library is an error, never a fallback.
"""
from .binding import (  # noqa: F401
    AttnTuning,
    KVCache,
    KvPool,
    PoolChange,
    SymphError,
    lib_path,
    load_library,
    kv_buffer_bytes,
    kv_pack,
    kv_unpack,
    kv_pack_layers,
    kv_unpack_layers,
    kv_pack_tail,
    kv_unpack_tail,
    kv_pack_units,
    kv_unpack_units,
    kv_append,
    prefix_prefill_attn,
    prefix_prefill_attn_workspace_bytes,
    prefix_prefill_attn_static,
    stage_to_host,
    stage_to_device,
    stage_layer_to_host,
    stage_layer_to_device,
    device_copy,
    mfma_reference,
    debug_check_tables,
    debug_attn_flags,
    status_string,
    EXPORTED_SYMBOLS,
)
