"""ctypes binding of the C ABI declared in include/fcdp.h.

Same names as the C entry points.  Pointers may be given as integers, as
objects with ``data_ptr()`` (torch tensors) or as ``None`` (NULL); streams as
integers, ``None`` (default stream) or objects with ``cuda_stream``
(torch.cuda.Stream).  Nothing here computes: it converts arguments, calls the
library and turns a non-zero status into ``FcdpError``.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

BF16 = 0
F32 = 1
SRC_DEVICE_SHARDS = 0
SRC_HOST_DMA = 1
SRC_HOST_ZEROCOPY = 2
SRC_DEVICE_RESIDENT = 3
SRC_HOST_SCATTER_DMA = 4
STORE_NONE = 0
STORE_DMA = 1
STORE_ZEROCOPY = 2
MAX_G = 64
STATIC_STAGING_BYTES = 32 << 20

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfcdp.so")
_lib: Optional[ctypes.CDLL] = None

STATUS_NAMES = {0: "FCDP_OK", 1: "FCDP_EINVAL", 2: "FCDP_ESIZE",
                3: "FCDP_EALIGN", 4: "FCDP_ENOTPINNED", 5: "FCDP_ESTATE",
                6: "FCDP_ENOMEM", 7: "FCDP_EHIP"}

# every symbol include/fcdp.h declares
EXPORTS = [
    "fcdp_layout_build", "fcdp_layout_destroy", "fcdp_layout_n_tensors",
    "fcdp_layout_G", "fcdp_layout_elem_size", "fcdp_layout_numel",
    "fcdp_layout_padded_numel", "fcdp_layout_shard_numel",
    "fcdp_layout_trainable_numel", "fcdp_layout_packed_numel",
    "fcdp_layout_offsets", "fcdp_layout_segments", "fcdp_layout_copy_plan",
    "fcdp_layout_prepare",
    "fcdp_materialize_layer", "fcdp_materialize_layer_static",
    "fcdp_cache_store", "fcdp_flatten_to_shards",
    "fcdp_cache_store_node_slice", "fcdp_materialize_layer_node_slice",
    "fcdp_reduce_grad_shard", "fcdp_reduce_trainable_shard",
    "fcdp_reduce_grad_shard_scaled", "fcdp_reduce_trainable_shard_scaled",
    "fcdp_pack_trainable", "fcdp_unpack_trainable", "fcdp_unpack_trainable_node_slice",
    "fcdp_host_cache_alloc", "fcdp_host_cache_free",
    "fcdp_cache_state_create", "fcdp_cache_state_destroy",
    "fcdp_cache_state_forward_source", "fcdp_cache_state_backward_source",
    "fcdp_cache_state_optimizer_step", "fcdp_cache_state_is_dirty",
    "fcdp_cache_state_mark_dirty",
    "fcdp_cache_state_set_tau", "fcdp_cache_state_place",
    "fcdp_cache_state_release", "fcdp_link_bytes",
    "fcdp_status_string", "fcdp_last_error", "fcdp_tuning_set",
    "fcdp_tuning_get", "fcdp_probe_copy", "fcdp_probe_reduce_stream", "fcdp_timing_enable",
    "fcdp_timing_collect",
]


class FcdpError(RuntimeError):
    def __init__(self, status: int, detail: str):
        self.status = status
        self.name = STATUS_NAMES.get(status, str(status))
        super().__init__("%s: %s" % (self.name, detail))


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Loads libfcdp.so; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            "libfcdp.so is missing at %s: build it with "
            "`python -m paper_2602_06499_amd.build` (there is no fallback)"
            % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    c = ctypes
    vp, i32, i64 = c.c_void_p, c.c_int32, c.c_int64
    lib.fcdp_layout_build.argtypes = [vp, vp, i32, i32, i32, i32, c.POINTER(vp)]
    lib.fcdp_layout_destroy.argtypes = [vp]
    lib.fcdp_layout_destroy.restype = None
    for nm in ("fcdp_layout_n_tensors", "fcdp_layout_G", "fcdp_layout_elem_size"):
        getattr(lib, nm).argtypes = [vp]
        getattr(lib, nm).restype = i32
    for nm in ("fcdp_layout_numel", "fcdp_layout_padded_numel",
               "fcdp_layout_shard_numel", "fcdp_layout_trainable_numel",
               "fcdp_layout_packed_numel"):
        getattr(lib, nm).argtypes = [vp]
        getattr(lib, nm).restype = i64
    lib.fcdp_layout_offsets.argtypes = [vp]
    lib.fcdp_layout_offsets.restype = c.POINTER(i64)
    lib.fcdp_layout_segments.argtypes = [vp, vp, i64]
    lib.fcdp_layout_segments.restype = i64
    lib.fcdp_layout_copy_plan.argtypes = [vp, i32, vp, i64]
    lib.fcdp_layout_copy_plan.restype = i64
    lib.fcdp_layout_prepare.argtypes = [vp]
    lib.fcdp_materialize_layer.argtypes = [vp, c.c_int, vp, vp, vp, vp, c.c_int, vp, vp]
    lib.fcdp_materialize_layer_static.argtypes = [vp, vp, vp, vp, vp]
    lib.fcdp_flatten_to_shards.argtypes = [vp, vp, vp, vp]
    lib.fcdp_cache_store.argtypes = [vp, vp, vp, c.c_int, vp, vp]
    lib.fcdp_cache_store_node_slice.argtypes = [vp, i32, i32, vp, vp, vp, vp]
    lib.fcdp_unpack_trainable_node_slice.argtypes = [vp, i32, i32, vp, vp, vp]
    lib.fcdp_materialize_layer_node_slice.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.fcdp_cache_state_set_tau.argtypes = [vp, c.c_double]
    lib.fcdp_cache_state_place.argtypes = [vp, i32, i64, i64, c.POINTER(i32)]
    lib.fcdp_cache_state_release.argtypes = [vp, i32]
    lib.fcdp_link_bytes.argtypes = [i32, c.POINTER(i64), c.POINTER(i64)]
    lib.fcdp_reduce_grad_shard.argtypes = [vp, i32, i64, i64, c.c_int, c.c_int, vp, vp]
    lib.fcdp_reduce_trainable_shard.argtypes = [vp, vp, i32, c.c_int, c.c_int, vp, vp]
    lib.fcdp_reduce_grad_shard_scaled.argtypes = [vp, i32, i64, i64, c.c_int, c.c_int, c.c_float, vp, vp]
    lib.fcdp_reduce_trainable_shard_scaled.argtypes = [vp, vp, i32, c.c_int, c.c_int, c.c_float, vp, vp]
    lib.fcdp_pack_trainable.argtypes = [vp, vp, vp, vp]
    lib.fcdp_unpack_trainable.argtypes = [vp, vp, vp, vp]
    lib.fcdp_host_cache_alloc.argtypes = [c.c_size_t, c.c_int, c.POINTER(vp), c.POINTER(vp)]
    lib.fcdp_host_cache_free.argtypes = [vp]
    lib.fcdp_cache_state_create.argtypes = [i32, c.POINTER(vp)]
    lib.fcdp_cache_state_destroy.argtypes = [vp]
    lib.fcdp_cache_state_destroy.restype = None
    lib.fcdp_cache_state_forward_source.argtypes = [vp, i32, i32, c.c_int, c.POINTER(c.c_int), c.POINTER(i32)]
    lib.fcdp_cache_state_backward_source.argtypes = [vp, i32, i32, c.c_int, c.POINTER(c.c_int)]
    lib.fcdp_cache_state_optimizer_step.argtypes = [vp]
    lib.fcdp_cache_state_is_dirty.argtypes = [vp, i32, i32]
    lib.fcdp_cache_state_mark_dirty.argtypes = [vp, i32, i32]
    lib.fcdp_cache_state_is_dirty.restype = i32
    lib.fcdp_status_string.argtypes = [c.c_int]
    lib.fcdp_status_string.restype = c.c_char_p
    lib.fcdp_last_error.argtypes = []
    lib.fcdp_last_error.restype = c.c_char_p
    lib.fcdp_tuning_set.argtypes = [c.c_char_p, i64]
    lib.fcdp_tuning_get.argtypes = [c.c_char_p]
    lib.fcdp_tuning_get.restype = i64
    lib.fcdp_probe_copy.argtypes = [vp, vp, c.c_size_t, vp]
    lib.fcdp_probe_reduce_stream.argtypes = [vp, vp, i32, i64, c.c_int, vp]
    lib.fcdp_timing_enable.argtypes = [i32]
    lib.fcdp_timing_collect.argtypes = [i32, c.POINTER(i64), c.POINTER(c.c_double)]
    _lib = lib
    return lib


def fcdp_last_error() -> str:
    return load_library().fcdp_last_error().decode()


def _check(status: int) -> None:
    if status != 0:
        raise FcdpError(status, fcdp_last_error())


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if hasattr(x, "dev"):           # HostCache
        return x.host
    raise TypeError("cannot take a pointer from %r" % type(x))


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    if isinstance(s, int):
        return s
    if hasattr(s, "cuda_stream"):
        return s.cuda_stream
    raise TypeError("cannot take a stream from %r" % type(s))


def pointer_array(xs: Sequence):
    """A reusable C array of pointers (saves the conversion on every call)."""
    return _ptr_array(list(xs))


def _ptr_array(xs: Optional[Sequence]):
    if xs is None:
        return None
    if isinstance(xs, ctypes.Array):
        return xs
    arr = (ctypes.c_void_p * max(len(xs), 1))()
    for i, x in enumerate(xs):
        arr[i] = _ptr(x)
    return arr


class Layout:
    """Owns an fcdp_layout handle."""

    def __init__(self, handle: int):
        self.handle = handle
        lib = load_library()
        self.n_tensors = lib.fcdp_layout_n_tensors(handle)
        self.G = lib.fcdp_layout_G(handle)
        self.elem_size = lib.fcdp_layout_elem_size(handle)
        self.numel = lib.fcdp_layout_numel(handle)
        self.padded_numel = lib.fcdp_layout_padded_numel(handle)
        self.shard_numel = lib.fcdp_layout_shard_numel(handle)
        self.trainable_numel = lib.fcdp_layout_trainable_numel(handle)
        self.packed_numel = lib.fcdp_layout_packed_numel(handle)
        p = lib.fcdp_layout_offsets(handle)
        self.offsets = [p[i] for i in range(self.n_tensors + 1)]

    def segments(self):
        lib = load_library()
        n = lib.fcdp_layout_segments(self.handle, None, 0)
        buf = (ctypes.c_int64 * (5 * max(n, 1)))()
        lib.fcdp_layout_segments(self.handle, buf, n)
        return [tuple(buf[i * 5 + k] for k in range(5)) for i in range(n)]

    def copy_plan(self, which: int):
        lib = load_library()
        n = lib.fcdp_layout_copy_plan(self.handle, which, None, 0)
        buf = (ctypes.c_int64 * (5 * max(n, 1)))()
        lib.fcdp_layout_copy_plan(self.handle, which, buf, n)
        return [tuple(buf[i * 5 + k] for k in range(5)) for i in range(n)]

    def prepare(self) -> None:
        _check(load_library().fcdp_layout_prepare(self.handle))

    def destroy(self) -> None:
        if self.handle:
            load_library().fcdp_layout_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def fcdp_layout_build(numel: Sequence[int], trainable: Optional[Sequence[int]],
                      G: int, elem_size: int = 2, pad_quantum: int = 64) -> Layout:
    lib = load_library()
    n = (ctypes.c_int64 * max(len(numel), 1))(*[int(k) for k in numel])
    tr = None
    if trainable is not None:
        tr = (ctypes.c_uint8 * max(len(trainable), 1))(*[int(bool(f)) for f in trainable])
    out = ctypes.c_void_p()
    _check(lib.fcdp_layout_build(n, tr, len(numel), G, elem_size, pad_quantum,
                                 ctypes.byref(out)))
    return Layout(out.value)


def fcdp_materialize_layer(layout: Layout, src: int, shard_ptrs, host_cache,
                           staging, tensor_ptrs, store_cache=STORE_NONE,
                           compute=None, copy=None) -> None:
    _check(load_library().fcdp_materialize_layer(
        layout.handle, src, _ptr_array(shard_ptrs), _ptr(host_cache),
        _ptr(staging), _ptr_array(tensor_ptrs), int(store_cache),
        _stream(compute), _stream(copy)))


def fcdp_materialize_layer_static(layout: Layout, host_cache, tensor_ptrs,
                                  compute=None, copy=None) -> None:
    _check(load_library().fcdp_materialize_layer_static(
        layout.handle, _ptr(host_cache), _ptr_array(tensor_ptrs),
        _stream(compute), _stream(copy)))


def fcdp_cache_store(layout: Layout, shard_ptrs, host_cache, store_mode=STORE_DMA,
                     compute=None, copy=None) -> None:
    _check(load_library().fcdp_cache_store(
        layout.handle, _ptr_array(shard_ptrs), _ptr(host_cache), int(store_mode),
        _stream(compute), _stream(copy)))


def fcdp_cache_store_node_slice(layout: Layout, first_shard: int, n_shards: int, shard_ptrs,
                                host_slice, compute=None, copy=None) -> None:
    _check(load_library().fcdp_cache_store_node_slice(
        layout.handle, first_shard, n_shards, _ptr_array(shard_ptrs), _ptr(host_slice),
        _stream(compute), _stream(copy)))


def fcdp_materialize_layer_node_slice(layout: Layout, first_shard: int, n_shards: int, shard_ptrs,
                                      host_slice, staging_slice, tensor_ptrs,
                                      compute=None, copy=None) -> None:
    _check(load_library().fcdp_materialize_layer_node_slice(
        layout.handle, first_shard, n_shards, _ptr_array(shard_ptrs), _ptr(host_slice),
        _ptr(staging_slice), _ptr_array(tensor_ptrs), _stream(compute), _stream(copy)))


def fcdp_link_bytes(reset: bool = False):
    """(stored, fetched) bytes sent over the host link through the library."""
    a, b = ctypes.c_int64(), ctypes.c_int64()
    _check(load_library().fcdp_link_bytes(int(reset), ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def fcdp_flatten_to_shards(layout: Layout, tensor_ptrs, shard_ptrs,
                           stream=None) -> None:
    _check(load_library().fcdp_flatten_to_shards(
        layout.handle, _ptr_array(tensor_ptrs), _ptr_array(shard_ptrs),
        _stream(stream)))


def fcdp_reduce_grad_shard(partial_ptrs, G: int, elem_offset: int, count: int,
                           in_dtype: int, out_dtype: int, out_shard,
                           stream=None) -> None:
    _check(load_library().fcdp_reduce_grad_shard(
        _ptr_array(partial_ptrs), G, elem_offset, count, in_dtype, out_dtype,
        _ptr(out_shard), _stream(stream)))


def fcdp_reduce_trainable_shard(layout: Layout, flat_grad_ptrs, rank: int,
                                in_dtype: int, out_dtype: int, out_shard,
                                stream=None) -> None:
    _check(load_library().fcdp_reduce_trainable_shard(
        layout.handle, _ptr_array(flat_grad_ptrs), rank, in_dtype, out_dtype,
        _ptr(out_shard), _stream(stream)))


def fcdp_reduce_grad_shard_scaled(partial_ptrs, G: int, elem_offset: int,
                                  count: int, in_dtype: int, out_dtype: int,
                                  scale: float, out_shard, stream=None) -> None:
    _check(load_library().fcdp_reduce_grad_shard_scaled(
        _ptr_array(partial_ptrs), G, elem_offset, count, in_dtype, out_dtype,
        scale, _ptr(out_shard), _stream(stream)))


def fcdp_reduce_trainable_shard_scaled(layout: Layout, flat_grad_ptrs, rank: int,
                                       in_dtype: int, out_dtype: int,
                                       scale: float, out_shard,
                                       stream=None) -> None:
    _check(load_library().fcdp_reduce_trainable_shard_scaled(
        layout.handle, _ptr_array(flat_grad_ptrs), rank, in_dtype, out_dtype,
        scale, _ptr(out_shard), _stream(stream)))


def fcdp_pack_trainable(layout: Layout, flat, packed, stream=None) -> None:
    _check(load_library().fcdp_pack_trainable(
        layout.handle, _ptr(flat), _ptr(packed), _stream(stream)))


def fcdp_unpack_trainable(layout: Layout, packed, flat, stream=None) -> None:
    _check(load_library().fcdp_unpack_trainable(
        layout.handle, _ptr(packed), _ptr(flat), _stream(stream)))


def fcdp_unpack_trainable_node_slice(layout: Layout, first_shard: int, n_shards: int, packed,
                                     flat_slice, stream=None) -> None:
    _check(load_library().fcdp_unpack_trainable_node_slice(
        layout.handle, first_shard, n_shards, _ptr(packed), _ptr(flat_slice), _stream(stream)))


class HostCache:
    """Pinned, device-mapped host buffer returned by fcdp_host_cache_alloc."""

    def __init__(self, host: int, dev: int, nbytes: int):
        self.host, self.dev, self.nbytes = host, dev, nbytes

    def numpy(self, dtype, count: Optional[int] = None, offset_bytes: int = 0):
        """A numpy view of the host memory (no copy)."""
        import numpy as np
        dt = np.dtype(dtype)
        if count is None:
            count = (self.nbytes - offset_bytes) // dt.itemsize
        buf = (ctypes.c_char * (count * dt.itemsize)).from_address(
            self.host + offset_bytes)
        return np.frombuffer(buf, dtype=dt, count=count)

    def free(self) -> None:
        if self.host:
            fcdp_host_cache_free(self.host)
            self.host = 0

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def fcdp_host_cache_alloc(nbytes: int, numa_node: int = -1) -> HostCache:
    host = ctypes.c_void_p()
    dev = ctypes.c_void_p()
    _check(load_library().fcdp_host_cache_alloc(
        nbytes, numa_node, ctypes.byref(host), ctypes.byref(dev)))
    return HostCache(host.value, dev.value, nbytes)


def fcdp_host_cache_free(host: int) -> None:
    _check(load_library().fcdp_host_cache_free(host))


class CacheState:
    """Dirty flags of Alg. 1 per (layer, class); class 0 frozen, 1 trainable."""

    def __init__(self, n_layers: int):
        out = ctypes.c_void_p()
        _check(load_library().fcdp_cache_state_create(n_layers, ctypes.byref(out)))
        self.handle = out.value

    def forward_source(self, layer: int, klass: int, host_mode: int):
        src = ctypes.c_int()
        store = ctypes.c_int32()
        _check(load_library().fcdp_cache_state_forward_source(
            self.handle, layer, klass, host_mode, ctypes.byref(src),
            ctypes.byref(store)))
        return src.value, bool(store.value)

    def backward_source(self, layer: int, klass: int, host_mode: int) -> int:
        src = ctypes.c_int()
        _check(load_library().fcdp_cache_state_backward_source(
            self.handle, layer, klass, host_mode, ctypes.byref(src)))
        return src.value

    def optimizer_step(self) -> None:
        _check(load_library().fcdp_cache_state_optimizer_step(self.handle))

    def set_tau(self, tau: float) -> None:
        _check(load_library().fcdp_cache_state_set_tau(self.handle, tau))

    def place(self, layer: int, used_bytes: int, total_bytes: int) -> bool:
        keep = ctypes.c_int32()
        _check(load_library().fcdp_cache_state_place(
            self.handle, layer, used_bytes, total_bytes, ctypes.byref(keep)))
        return bool(keep.value)

    def release(self, layer: int) -> None:
        _check(load_library().fcdp_cache_state_release(self.handle, layer))

    def mark_dirty(self, layer: int, klass: int) -> None:
        _check(load_library().fcdp_cache_state_mark_dirty(self.handle, layer, klass))

    def is_dirty(self, layer: int, klass: int) -> int:
        return load_library().fcdp_cache_state_is_dirty(self.handle, layer, klass)

    def __del__(self):
        try:
            if self.handle:
                load_library().fcdp_cache_state_destroy(self.handle)
                self.handle = None
        except Exception:
            pass


def fcdp_tuning_set(name: str, value: int) -> None:
    _check(load_library().fcdp_tuning_set(name.encode(), value))


def fcdp_tuning_get(name: str) -> int:
    return load_library().fcdp_tuning_get(name.encode())


KERNEL_UNFLATTEN = 0
KERNEL_UNFLATTEN_ZEROCOPY = 1
KERNEL_FLATTEN = 2
KERNEL_REDUCE = 3
KERNEL_PACK = 4
KERNEL_UNPACK = 5
KERNEL_STORE_ZEROCOPY = 6
KERNEL_PROBE_COPY = 7
KERNEL_REDUCE_TRAINABLE = 8
KERNEL_PROBE_STREAM = 9


def fcdp_timing_enable(capacity: int) -> None:
    _check(load_library().fcdp_timing_enable(capacity))


def fcdp_timing_collect(kind: int):
    """(launches, total_ms) of the timed launches of one kernel kind."""
    n = ctypes.c_int64()
    ms = ctypes.c_double()
    _check(load_library().fcdp_timing_collect(kind, ctypes.byref(n), ctypes.byref(ms)))
    return n.value, ms.value


def fcdp_probe_copy(dst, src, nbytes: int, stream=None) -> None:
    _check(load_library().fcdp_probe_copy(_ptr(dst), _ptr(src), nbytes,
                                          _stream(stream)))


def fcdp_probe_reduce_stream(dst, src, G: int, count: int, out_dtype: int, stream=None) -> None:
    _check(load_library().fcdp_probe_reduce_stream(_ptr(dst), _ptr(src), G, count, out_dtype,
                                                   _stream(stream)))
