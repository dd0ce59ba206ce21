"""CPU oracle for the FCDP per-layer hot path -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The product (the HIP library and its
binding under ``paper_2602_06499_amd/``) never does, and this package never
imports the product.

The arithmetic lives in ``fcdp_oracle.c`` (plain scalar C, compiled here with
gcc); this module only marshals numpy arrays into it.  bf16 data is carried as
``numpy.uint16`` bit patterns, fp32 as ``numpy.float32``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fcdp_oracle.c")
_SO = os.path.join(_HERE, "libfcdp_oracle.so")

CFLAGS = ["-O2", "-std=c11", "-Wall", "-Wextra", "-ffp-contract=off",
          "-fno-fast-math", "-shared", "-fPIC"]

BF16 = 0
F32 = 1


def build(force: bool = False) -> str:
    """Compile fcdp_oracle.c with gcc; returns the path of the shared object."""
    if force or not os.path.exists(_SO) or \
            os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        tmp = _SO + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC])
        os.replace(tmp, _SO)
    return _SO


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.fcdp_oracle_segments.restype = ctypes.c_int64
        _lib.fcdp_oracle_bf16_rne.restype = ctypes.c_uint16
        _lib.fcdp_oracle_bf16_rne.argtypes = [ctypes.c_float]
    return _lib


def _i64(a: Sequence[int]) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int64))


def _p(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def _ptr_array(arrs: Sequence[np.ndarray]):
    return (ctypes.c_void_p * max(len(arrs), 1))(
        *[a.ctypes.data for a in arrs])


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError("oracle %s: invalid argument" % what)


def _c(a: np.ndarray) -> np.ndarray:
    if not a.flags["C_CONTIGUOUS"]:
        raise ValueError("oracle inputs must be C-contiguous")
    return a


def layout(numel: Sequence[int], G: int, q: int = 64) -> dict:
    """Offset table: off (T+1), N, N_pad, S."""
    n = _i64(numel)
    off = np.zeros(len(n) + 1, dtype=np.int64)
    N = ctypes.c_int64()
    Np = ctypes.c_int64()
    S = ctypes.c_int64()
    _check(lib().fcdp_oracle_layout(_p(n), ctypes.c_int32(len(n)),
                                    ctypes.c_int32(G), ctypes.c_int32(q),
                                    _p(off), ctypes.byref(N),
                                    ctypes.byref(Np), ctypes.byref(S)),
           "layout")
    return {"off": off, "N": N.value, "N_pad": Np.value, "S": S.value}


def flatten(tensors: Sequence[np.ndarray], G: int, q: int = 64) -> np.ndarray:
    """Padded flat image of a layer (zero tail padding)."""
    dt = tensors[0].dtype if len(tensors) else np.dtype(np.uint16)
    n = _i64([t.size for t in tensors])
    lay = layout(n, G, q)
    flat = np.empty(lay["N_pad"], dtype=dt)
    flat.view(np.uint8)[:] = 0xA5  # poison: the oracle must write every byte
    ts = [_c(t) for t in tensors]
    _check(lib().fcdp_oracle_flatten(_ptr_array(ts), _p(n),
                                     ctypes.c_int32(len(n)),
                                     ctypes.c_int32(G), ctypes.c_int32(q),
                                     ctypes.c_int32(dt.itemsize), _p(flat)),
           "flatten")
    return flat


def split(flat: np.ndarray, G: int) -> List[np.ndarray]:
    """G equal rank shards of the padded flat image."""
    if flat.size % G:
        raise ValueError("flat size not divisible by G")
    S = flat.size // G
    shards = [np.empty(S, dtype=flat.dtype) for _ in range(G)]
    _check(lib().fcdp_oracle_split(_p(_c(flat)), ctypes.c_int64(S),
                                   ctypes.c_int32(G),
                                   ctypes.c_int32(flat.dtype.itemsize),
                                   _ptr_array(shards)), "split")
    return shards


def _alloc_tensors(numel, dt) -> List[np.ndarray]:
    out = []
    for k in numel:
        a = np.empty(int(k), dtype=dt)
        a.view(np.uint8)[:] = 0x5A
        out.append(a)
    return out


def materialize_from_shards(shards: Sequence[np.ndarray],
                            numel: Sequence[int]) -> List[np.ndarray]:
    """Full per-tensor parameters from the G rank shards."""
    n = _i64(numel)
    dt = shards[0].dtype
    S = shards[0].size
    out = _alloc_tensors(n, dt)
    sh = [_c(s) for s in shards]
    _check(lib().fcdp_oracle_materialize_from_shards(
        _ptr_array(sh), ctypes.c_int64(S), ctypes.c_int32(len(sh)), _p(n),
        ctypes.c_int32(len(n)), ctypes.c_int32(dt.itemsize),
        _ptr_array(out)), "materialize_from_shards")
    return out


def materialize_from_flat(flat: np.ndarray,
                          numel: Sequence[int]) -> List[np.ndarray]:
    """Full per-tensor parameters from the cached padded flat image."""
    n = _i64(numel)
    if int(n.sum()) > flat.size:
        raise ValueError("flat image smaller than the layer")
    out = _alloc_tensors(n, flat.dtype)
    _check(lib().fcdp_oracle_materialize_from_flat(
        _p(_c(flat)), _p(n), ctypes.c_int32(len(n)),
        ctypes.c_int32(flat.dtype.itemsize), _ptr_array(out)),
        "materialize_from_flat")
    return out


def cache_store(shards: Sequence[np.ndarray]) -> np.ndarray:
    """Host-cache image of a layer: the shards in rank order."""
    dt = shards[0].dtype
    S = shards[0].size
    H = np.empty(S * len(shards), dtype=dt)
    sh = [_c(s) for s in shards]
    _check(lib().fcdp_oracle_cache_store(
        _ptr_array(sh), ctypes.c_int64(S), ctypes.c_int32(len(sh)),
        ctypes.c_int32(dt.itemsize), _p(H)), "cache_store")
    return H


def segments(numel: Sequence[int], G: int, q: int = 64) -> np.ndarray:
    """(t, r, dst_off, src_off, len) rows of the tensor x shard overlaps."""
    n = _i64(numel)
    cap = len(n) + G + 1
    rows = np.zeros((cap, 5), dtype=np.int64)
    cnt = lib().fcdp_oracle_segments(_p(n), ctypes.c_int32(len(n)),
                                     ctypes.c_int32(G), ctypes.c_int32(q),
                                     _p(rows), ctypes.c_int64(cap))
    assert cnt <= cap
    return rows[:cnt].copy()


def bf16_rne(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round to nearest even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    lib().fcdp_oracle_bf16_rne_array(_p(x), ctypes.c_int64(x.size), _p(out))
    return out


def reduce(partials: Sequence[np.ndarray], elem_offset: int, count: int,
           out_dtype: int, scale=None) -> np.ndarray:
    """Rank-order fp32 sum of G partial gradient slices.

    partials: G arrays, float32 (fp32 input) or uint16 (bf16 input).
    out_dtype: BF16 -> uint16 result, F32 -> float32 result.
    scale: None for the plain sum; a float multiplies the finished sum once
    in fp32 (1/G gives the mean).
    """
    dt = partials[0].dtype
    if dt == np.float32:
        in_dtype = F32
    elif dt == np.uint16:
        in_dtype = BF16
    else:
        raise ValueError("partials must be float32 or uint16 (bf16 bits)")
    for p in partials:
        if p.dtype != dt or elem_offset + count > p.size or elem_offset < 0:
            raise ValueError("partial too small or dtype mismatch")
    out = np.empty(count, dtype=np.float32 if out_dtype == F32 else np.uint16)
    ps = [_c(p) for p in partials]
    if scale is None:
        _check(lib().fcdp_oracle_reduce(
            _ptr_array(ps), ctypes.c_int32(len(ps)),
            ctypes.c_int64(elem_offset), ctypes.c_int64(count),
            ctypes.c_int32(in_dtype), ctypes.c_int32(out_dtype), _p(out)),
            "reduce")
    else:
        _check(lib().fcdp_oracle_reduce_scaled(
            _ptr_array(ps), ctypes.c_int32(len(ps)),
            ctypes.c_int64(elem_offset), ctypes.c_int64(count),
            ctypes.c_int32(in_dtype), ctypes.c_int32(out_dtype),
            ctypes.c_float(scale), _p(out)), "reduce_scaled")
    return out


def packed_numel(numel: Sequence[int], trainable: Sequence[int], G: int,
                 q: int = 64) -> int:
    nt = sum(int(k) for k, f in zip(numel, trainable) if f)
    Q = G * q
    return ((nt + Q - 1) // Q) * Q


def pack(flat: np.ndarray, numel: Sequence[int], trainable: Sequence[int],
         G: int, q: int = 64) -> np.ndarray:
    """Trainable tensors' flat ranges, concatenated, zero-padded to G*q."""
    n = _i64(numel)
    tr = np.ascontiguousarray(np.asarray(trainable, dtype=np.uint8))
    out = np.empty(packed_numel(numel, trainable, G, q), dtype=flat.dtype)
    out.view(np.uint8)[:] = 0xA5
    nt = ctypes.c_int64()
    _check(lib().fcdp_oracle_pack(
        _p(_c(flat)), _p(n), _p(tr), ctypes.c_int32(len(n)),
        ctypes.c_int32(G), ctypes.c_int32(q),
        ctypes.c_int32(flat.dtype.itemsize), _p(out), ctypes.byref(nt)),
        "pack")
    return out


def unpack(packed: np.ndarray, flat: np.ndarray, numel: Sequence[int],
           trainable: Sequence[int]) -> None:
    """Write the packed trainable values back into flat, in place."""
    n = _i64(numel)
    tr = np.ascontiguousarray(np.asarray(trainable, dtype=np.uint8))
    if packed.dtype != flat.dtype:
        raise ValueError("dtype mismatch")
    _check(lib().fcdp_oracle_unpack(
        _p(_c(packed)), _p(n), _p(tr), ctypes.c_int32(len(n)),
        ctypes.c_int32(flat.dtype.itemsize), _p(_c(flat))), "unpack")


def reduce_trainable(flat_partials: Sequence[np.ndarray], numel: Sequence[int],
                     trainable: Sequence[int], G: int, rank: int,
                     out_dtype: int, q: int = 64, scale=None) -> np.ndarray:
    """This rank's shard of the summed trainable gradients.

    The composition of two definitions above: every rank's flat gradient is
    packed (trainable ranges in tensor order, zero tail), then the packed
    buffers are summed in rank order over this rank's slice.
    """
    packed = [pack(p, numel, trainable, G, q) for p in flat_partials]
    Sp = packed[0].size // G
    return reduce(packed, rank * Sp, Sp, out_dtype, scale)
