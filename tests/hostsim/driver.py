"""Runs the library's entry points in a host build under ASan + UBSan.

Started by tests/test_hostsim_sanitizers.py as a child process with the
sanitizer runtime preloaded; argv[1] is the host build of the library (the
product's sources compiled against the stand-in HIP runtime in this folder,
where device memory is host memory and a launch runs every thread of the grid
in turn).  Every buffer handed to the library is an allocation of exactly the
documented size, so a read or write one byte outside it is an ASan report, and
results are compared with the CPU oracle like the GPU parity tests do.  This
checks the index arithmetic of the kernels and the host code around them; it
says nothing about the GPU's execution, which the GPU tests cover.
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from paper_2602_06499_amd import binding  # noqa: E402

binding._LIB_PATH = sys.argv[1]

import oracle  # noqa: E402
import paper_2602_06499_amd as fcdp  # noqa: E402
from paper_2602_06499_amd import synth  # noqa: E402

STREAM_A, STREAM_B = 0x1000, 0x2000     # opaque to the stand-in runtime


class Buf:
    """nbytes of host memory that end where their allocation ends; `offset`
    shifts the start off 16-byte alignment."""

    def __init__(self, nbytes, offset=0, fill=0xC3):
        self.raw = np.full(nbytes + offset, fill, np.uint8)
        self.a = self.raw[offset:]

    def data_ptr(self):
        return self.a.ctypes.data

    def view(self, dt):
        k = np.dtype(dt).itemsize
        return self.a[:self.a.size // k * k].view(dt)


def dev(x, offset=0):
    b = Buf(x.nbytes, offset)
    b.a[:] = np.ascontiguousarray(x).view(np.uint8).reshape(-1)
    return b


def rand_tensors(seed, sizes, dt):
    g = synth.rng(0, seed, synth.KIND_MISC, 33)
    return [g.integers(0, int(np.iinfo(dt).max) + 1, size=k, dtype=dt) for k in sizes]


def check_layer(name, sizes, G, esz, offset):
    dt = np.uint16 if esz == 2 else np.uint32
    tensors = rand_tensors(len(sizes) + 7 * G, sizes, dt)
    flat = oracle.flatten(tensors, G)
    shards = oracle.split(flat, G)
    want = oracle.materialize_from_shards(shards, sizes)
    L = fcdp.fcdp_layout_build(sizes, None, G, esz)
    L.prepare()
    S, Np = L.shard_numel, L.padded_numel
    d_shards = [dev(s, offset) for s in shards]
    H = fcdp.fcdp_host_cache_alloc(max(Np * esz, 16))
    for store in (fcdp.STORE_DMA, fcdp.STORE_ZEROCOPY):
        H.numpy(np.uint8)[:] = 0x77
        outs = [Buf(k * esz, offset) for k in sizes]
        fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, d_shards, H, None,
                                    outs, store, STREAM_A, STREAM_B)
        for t, w in enumerate(want):
            assert np.array_equal(outs[t].view(dt), w), (name, "shards", t)
        assert np.array_equal(H.numpy(dt, Np), flat), (name, "store", store)
    back = [Buf(S * esz, offset) for _ in range(G)]
    fcdp.fcdp_flatten_to_shards(L, outs, back, None)
    for r in range(G):
        assert np.array_equal(back[r].view(dt), shards[r]), (name, "flatten", r)
    for mode in (fcdp.SRC_HOST_DMA, fcdp.SRC_HOST_ZEROCOPY,
                 fcdp.SRC_HOST_SCATTER_DMA):
        outs = [Buf(k * esz, offset) for k in sizes]
        staging = Buf(Np * esz) if mode == fcdp.SRC_HOST_DMA else None
        fcdp.fcdp_materialize_layer(L, mode, None, H, staging, outs,
                                    fcdp.STORE_NONE, STREAM_A, STREAM_B)
        for t, w in enumerate(want):
            assert np.array_equal(outs[t].view(dt), w), (name, mode, t)
    if Np * esz <= fcdp.STATIC_STAGING_BYTES:
        # the allocation-free staged fetch: same tensors out of the static array
        outs = [Buf(k * esz, offset) for k in sizes]
        fcdp.fcdp_materialize_layer_static(L, H, outs, STREAM_A, STREAM_B)
        for t, w in enumerate(want):
            assert np.array_equal(outs[t].view(dt), w), (name, "static", t)
    # one GPU's share of a node: every split of the G shards into equal parts that has
    # more than one part, first and last part; exactly sized slice buffers
    for g in [d for d in (2, 3, 4, 8) if G % d == 0 and S > 0]:
        n = G // g
        for first in sorted({0, G - n}):
            Hs = fcdp.fcdp_host_cache_alloc(n * S * esz)
            own = [d_shards[r] if first <= r < first + n else None for r in range(G)]
            fcdp.fcdp_cache_store_node_slice(L, first, n, own, Hs, STREAM_A, STREAM_B)
            assert np.array_equal(Hs.numpy(dt, n * S), flat[first * S:(first + n) * S]), (name, "slice store", g, first)
            peers = [None if first <= r < first + n else d_shards[r] for r in range(G)]
            outs = [Buf(k * esz, offset) for k in sizes]
            stg = Buf(n * S * esz)
            fcdp.fcdp_materialize_layer_node_slice(L, first, n, peers, Hs, stg, outs, STREAM_A, STREAM_B)
            for t, w in enumerate(want):
                assert np.array_equal(outs[t].view(dt), w), (name, "slice fetch", g, first, t)
            Hs.free()
    H.free()
    L.destroy()


def check_reduce(G, count, e0, in_dt, out_dt, offset, scale=None):
    g = synth.rng(0, G * 1000 + count % 997, synth.KIND_GRAD, 9)
    n = e0 + count
    parts = []
    for _ in range(G):
        x = (g.standard_normal(n, dtype=np.float32)
             * np.exp2(g.integers(-20, 20, size=n)).astype(np.float32))
        parts.append(synth.to_bf16_bits(x) if in_dt == oracle.BF16 else x)
    want = oracle.reduce(parts, e0, count, out_dt, scale)
    d_parts = [dev(p, offset) for p in parts]
    osz = 4 if out_dt == oracle.F32 else 2
    d_out = Buf(count * osz, offset)
    if scale is None:
        fcdp.fcdp_reduce_grad_shard(d_parts, G, e0, count, in_dt, out_dt, d_out, None)
    else:
        fcdp.fcdp_reduce_grad_shard_scaled(d_parts, G, e0, count, in_dt, out_dt, scale,
                                           d_out, None)
    got = d_out.view(np.uint32 if osz == 4 else np.uint16)
    assert np.array_equal(got, want.view(got.dtype)), ("reduce", G, count, e0, in_dt, out_dt)


def check_peft(name, sizes, tr, G, esz):
    dt = np.uint16 if esz == 2 else np.uint32
    tensors = rand_tensors(len(sizes) + 13 * G, sizes, dt)
    flat = oracle.flatten(tensors, G)
    L = fcdp.fcdp_layout_build(sizes, tr, G, esz)
    L.prepare()
    Pn = L.packed_numel
    want = oracle.pack(flat, sizes, tr, G)
    assert Pn == want.size
    d_flat = dev(flat)
    d_packed = Buf(max(Pn * esz, 16))
    fcdp.fcdp_pack_trainable(L, d_flat, d_packed, None)
    assert np.array_equal(d_packed.view(dt)[:Pn], want), (name, "pack")
    g = synth.rng(0, len(sizes), synth.KIND_MISC, 77)
    newp = g.integers(0, int(np.iinfo(dt).max) + 1, size=Pn, dtype=dt)
    ref = flat.copy()
    oracle.unpack(newp, ref, sizes, tr)
    d_new = dev(newp) if Pn else Buf(16)
    fcdp.fcdp_unpack_trainable(L, d_new, d_flat, None)
    assert np.array_equal(d_flat.view(dt), ref), (name, "unpack")
    # the same unpack clipped to a node slice, into exactly sized slice buffers
    S = L.shard_numel
    for gg in [d for d in (2, 4) if G % d == 0 and S > 0]:
        n = G // gg
        for first in range(0, G, n):
            d_slice = dev(flat[first * S:(first + n) * S])
            fcdp.fcdp_unpack_trainable_node_slice(L, first, n, d_new, d_slice, None)
            assert np.array_equal(d_slice.view(dt), ref[first * S:(first + n) * S]), (name, "slice unpack", gg, first)
    if esz != 2 or Pn == 0:
        return
    # fused pack + reduce from G flat fp32 / bf16 gradients
    for in_dt, out_dt in ((oracle.F32, oracle.F32), (oracle.BF16, oracle.BF16),
                          (oracle.F32, oracle.BF16)):
        n = L.padded_numel
        parts = []
        for r in range(G):
            x = synth.rng(0, r, synth.KIND_GRAD, 5).standard_normal(n, dtype=np.float32)
            parts.append(synth.to_bf16_bits(x) if in_dt == oracle.BF16 else x)
        for rank in sorted({0, G // 2, G - 1}):
            d_parts = [dev(p) for p in parts]
            osz = 4 if out_dt == oracle.F32 else 2
            for scale in (None, float(np.float32(-1.0 / G))):
                want = oracle.reduce_trainable(parts, sizes, tr, G, rank, out_dt, scale=scale)
                d_out = Buf(want.size * osz)
                if scale is None:
                    fcdp.fcdp_reduce_trainable_shard(L, d_parts, rank, in_dt, out_dt, d_out, None)
                else:
                    fcdp.fcdp_reduce_trainable_shard_scaled(L, d_parts, rank, in_dt, out_dt,
                                                            scale, d_out, None)
                got = d_out.view(np.uint32 if osz == 4 else np.uint16)
                assert np.array_equal(got, want.view(got.dtype)), (name, "reduce_trainable", rank, scale)


def planted_short_output():
    """A caller's mistake on purpose: the last output tensor is 2 bytes short.
    The run must die with an ASan report, which shows that the harness sees an
    access past a buffer's end."""
    sizes, G = [1000, 24], 2
    tensors = rand_tensors(1, sizes, np.uint16)
    shards = oracle.split(oracle.flatten(tensors, G), G)
    L = fcdp.fcdp_layout_build(sizes, None, G, 2)
    outs = [Buf(2000), Buf(46)]
    fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, [dev(s) for s in shards],
                                None, None, outs, fcdp.STORE_NONE, None, None)
    print("planted mistake went unseen", flush=True)


def main():
    if len(sys.argv) > 2 and sys.argv[2] == "--plant-short-output":
        planted_short_output()
        return
    n = 0
    layer_cases = [
        ("tiny_padding_only_shards", [3, 0, 1], 8, 2),
        ("single_element", [1], 4, 2),
        ("zeros_and_one", [0, 0, 5, 0], 3, 4),
        ("odd_multi_tile", [30001, 7, 65537, 13107], 3, 2),
        ("many_tensors", [(i * 37) % 501 for i in range(600)], 5, 2),
    ]
    for G in (1, 2, 3, 8, 64):
        for k, esz in enumerate((2, 4)):
            sizes = synth.random_layer(4000 + G * 3 + k, T=7 + G % 5, max_numel=20000)
            layer_cases.append(("rand_G%d_e%d" % (G, esz), sizes, G, esz))
    cfg = synth.CONFIGS["gpt2_small_g4"]
    layer_cases.append((cfg.name, list(cfg.numel), cfg.G, 2))
    for name, sizes, G, esz in layer_cases:
        print("layer", name, flush=True)
        check_layer(name, sizes, G, esz, 0)     # the ABI wants 16-byte aligned bases
        n += 1
    fcdp.fcdp_tuning_set("debug_poison", 1)     # the poison fills, same results
    for name, sizes, G, esz in layer_cases[:6]:
        print("layer (poison)", name, flush=True)
        check_layer(name, sizes, G, esz, 0)
        n += 1
    fcdp.fcdp_tuning_set("debug_poison", 0)
    reduce_cases = [(1, 1000, 0), (2, 4099, 0), (3, 7001, 5), (7, 3333, 3),
                    (8, 30007, 0), (9, 1234, 1), (15, 5000, 2), (16, 6553, 0),
                    (17, 4000, 7), (33, 2049, 0), (64, 3001, 11), (5, 3, 0),
                    (5, 0, 0),
                    # long enough for the rule to pick the phased reduce (the stand-in device
                    # has 4 compute units: a launch holds 16 waves x 104 steps x 256 elements
                    # = 425 984): two waves per SIMD, two launches, the unaligned fallback,
                    # one wave per SIMD
                    (9, 270001, 0), (3, 600007, 0), (3, 600007, 1), (8, 330003, 0), (16, 700001, 8)]
    # the phased reduce forced from 8 steps per wave on: both shapes, short runs, a run of
    # 43 steps per wave (started at step w mod 43), and every run rotated
    forced_cases = [(2, 66000, 4, 0, 1), (8, 66003, 0, 0, 1), (16, 140001, 8, 0, 1), (8, 500009, 0, 0, 1),
                    (8, 43 * 16 * 256 - 100, 0, 1, 1), (8, 43 * 16 * 256 - 100, 0, 2, 1),
                    (24, 300003, 0, 0, 2), (11, 250001, 4, 0, 2), (8, 300003, 0, 0, 2)]
    for G, count, e0 in reduce_cases:
        for in_dt, out_dt in ((oracle.F32, oracle.F32), (oracle.F32, oracle.BF16),
                              (oracle.BF16, oracle.BF16), (oracle.BF16, oracle.F32)):
            print("reduce", G, count, e0, in_dt, out_dt, flush=True)
            check_reduce(G, count, e0, in_dt, out_dt, 0)
            check_reduce(G, count, e0, in_dt, out_dt, 0, float(np.float32(1.0 / G)))
            n += 2
    for G, count, e0, waves, rotate in forced_cases:
        fcdp.fcdp_tuning_set("reduce_phased", 1)
        fcdp.fcdp_tuning_set("reduce_phase_waves", waves)
        fcdp.fcdp_tuning_set("reduce_phase_rotate", rotate)
        for in_dt, out_dt in ((oracle.F32, oracle.F32), (oracle.F32, oracle.BF16),
                              (oracle.BF16, oracle.BF16), (oracle.BF16, oracle.F32)):
            print("reduce, phased forced", G, count, e0, waves, rotate, in_dt, out_dt, flush=True)
            check_reduce(G, count, e0, in_dt, out_dt, 0)
            if in_dt == oracle.F32:                 # bf16 steps are twice as long: some cases are too short
                assert fcdp.fcdp_tuning_get("last_reduce_shape") != 0
            n += 1
        fcdp.fcdp_tuning_set("reduce_phased", 2)
        fcdp.fcdp_tuning_set("reduce_phase_waves", 0)
        fcdp.fcdp_tuning_set("reduce_phase_rotate", 1)
    for G, tiles in ((1, 2), (5, 7), (8, 3), (19, 2), (64, 1)):
        print("calibration stream", G, tiles, flush=True)
        src = synth.rng(0, G, synth.KIND_GRAD, 3).standard_normal((tiles, G, 1024), dtype=np.float32)
        parts = [np.ascontiguousarray(src[:, r, :]).reshape(-1) for r in range(G)]
        for out_dt in (oracle.F32, oracle.BF16):
            d_out = Buf(tiles * 1024 * (4 if out_dt == oracle.F32 else 2))
            fcdp.fcdp_probe_reduce_stream(d_out, dev(src), G, tiles * 1024, out_dt, None)
            got = d_out.view(np.uint32 if out_dt == oracle.F32 else np.uint16)
            assert np.array_equal(got, oracle.reduce(parts, 0, tiles * 1024, out_dt).view(got.dtype)), (G, tiles)
        n += 1
    for name, sizes, tr, G, esz in PEFT_CASES():
        print("peft", name, flush=True)
        check_peft(name, sizes, tr, G, esz)
        n += 1
    # the numa_node argument of the host cache allocation: every accepted value gives a
    # usable buffer (the policy is best effort), the out-of-range one is an argument error
    for node in (-1, 0, 1, 63, 1023):
        H = fcdp.fcdp_host_cache_alloc(4096, numa_node=node)
        note = fcdp.fcdp_last_error()
        assert note == "" or "NUMA policy refused" in note or "no NUMA policy call" in note, note
        H.numpy(np.uint8)[:] = 7
        H.free()
        n += 1
    for bad in (1024, 1 << 20):
        try:
            fcdp.fcdp_host_cache_alloc(4096, numa_node=bad)
        except fcdp.FcdpError as e:
            assert e.name == "FCDP_EINVAL", e
        else:
            raise AssertionError("numa_node %d was accepted" % bad)
    print("hostsim ok: %d cases" % n, flush=True)


def PEFT_CASES():
    cfg = synth.CONFIGS["gpt2_small_g4"]
    return [
        ("lora_like", [4096, 64, 64, 4096, 128, 128, 9000], [0, 1, 1, 0, 1, 1, 0], 4, 2),
        ("none_trainable", [100, 200], [0, 0], 2, 2),
        ("all_trainable_odd", [333, 1, 0, 4097], [1, 1, 1, 1], 3, 2),
        ("alternating_f32", [17, 1000, 3, 2049, 5], [1, 0, 1, 0, 1], 8, 4),
        ("gpt2_bias_only", list(cfg.numel),
         [1 if k < 10000 else 0 for k in cfg.numel], cfg.G, 2),
    ]


if __name__ == "__main__":
    main()
