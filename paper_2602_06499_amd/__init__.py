"""FCDP per-layer hot path for one MI355X: Python binding of libfcdp.so.

The binding only marshals arguments; every step of the path runs in the HIP
library.  Importing the package does not load the library; the first call
does, and raises if it has not been built (there is no CPU fallback).
"""
from .binding import (  # noqa: F401
    BF16, F32, SRC_DEVICE_SHARDS, SRC_HOST_DMA, SRC_HOST_ZEROCOPY, MAX_G,
    SRC_DEVICE_RESIDENT, SRC_HOST_SCATTER_DMA, fcdp_cache_store, fcdp_link_bytes,
    STORE_NONE, STORE_DMA, STORE_ZEROCOPY,
    FcdpError, Layout, CacheState, HostCache,
    fcdp_layout_build, fcdp_materialize_layer, fcdp_flatten_to_shards,
    fcdp_materialize_layer_static, STATIC_STAGING_BYTES,
    fcdp_cache_store_node_slice, fcdp_materialize_layer_node_slice, fcdp_unpack_trainable_node_slice,
    fcdp_reduce_grad_shard, fcdp_reduce_trainable_shard, fcdp_pack_trainable, fcdp_unpack_trainable,
    fcdp_reduce_grad_shard_scaled, fcdp_reduce_trainable_shard_scaled,
    fcdp_host_cache_alloc, fcdp_host_cache_free, fcdp_tuning_set,
    fcdp_tuning_get, fcdp_probe_copy, fcdp_last_error, load_library,
    library_path, pointer_array, fcdp_timing_enable, fcdp_timing_collect,
    KERNEL_UNFLATTEN, KERNEL_UNFLATTEN_ZEROCOPY, KERNEL_FLATTEN, KERNEL_REDUCE,
    KERNEL_PACK, KERNEL_UNPACK, KERNEL_STORE_ZEROCOPY, KERNEL_PROBE_COPY, KERNEL_REDUCE_TRAINABLE,
    KERNEL_PROBE_STREAM, fcdp_probe_reduce_stream,
)
