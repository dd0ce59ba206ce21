"""CPU tests of the library's host side: it loads, exports what the header
declares, builds the same offset table and segment list as the oracle, its
copy plans (interpreted here with numpy) reproduce the oracle's results, its
dirty-state flags follow the Alg. 1 replay, and bad arguments come back as
status codes before anything is enqueued."""
import ctypes
import os
import re

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import oracle
from oracle import alg1
import paper_2602_06499_amd as fcdp
from paper_2602_06499_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _rand_tensors(seed, sizes, dtype=np.uint16):
    g = synth.rng(0, seed, synth.KIND_MISC, 31)
    info = np.iinfo(dtype)
    return [g.integers(0, int(info.max) + 1, size=k, dtype=dtype) for k in sizes]


def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "fcdp.h")) as f:
        text = f.read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(fcdp_[a-z_0-9A-Z]+)\s*\(", text))
    assert declared == set(binding.EXPORTS)
    lib = fcdp.load_library()
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert os.path.dirname(fcdp.library_path()).endswith("paper_2602_06499_amd")


LAYOUTS = [(synth.random_layer(2000 + i, T=3 + i % 9, max_numel=3000), G, esz)
           for i, (G, esz) in enumerate([(1, 2), (2, 2), (3, 4), (4, 2), (5, 2), (8, 4),
                                         (16, 2), (32, 2), (64, 2), (7, 4)])]
LAYOUTS += [([3, 0, 1], 8, 2), ([0, 0], 4, 2), ([1], 1, 2), ([70000, 5, 65536, 9], 3, 2)]


@pytest.mark.parametrize("sizes,G,esz", LAYOUTS)
def test_layout_matches_oracle(sizes, G, esz):
    tr = [(t * 7 + G) % 3 == 0 for t in range(len(sizes))]
    L = fcdp.fcdp_layout_build(sizes, tr, G, esz)
    lay = oracle.layout(sizes, G)
    assert (L.numel, L.padded_numel, L.shard_numel) == (lay["N"], lay["N_pad"], lay["S"])
    assert L.offsets == lay["off"].tolist()
    assert L.n_tensors == len(sizes) and L.G == G and L.elem_size == esz
    assert L.trainable_numel == sum(k for k, f in zip(sizes, tr) if f)
    assert L.packed_numel == oracle.packed_numel(sizes, tr, G)
    segs = np.array(L.segments(), dtype=np.int64).reshape(-1, 5)
    assert np.array_equal(segs, oracle.segments(sizes, G))


def _run_plan(plan, srcs, dsts):
    """Interpret a copy plan on host byte buffers (the kernel's contract)."""
    for si, so, di, do, nb in plan:
        assert nb > 0 and nb % 2 == 0
        d = dsts[di]
        assert 0 <= do and do + nb <= d.size, "destination range out of bounds"
        if si < 0:
            d[do:do + nb] = 0
        else:
            s = srcs[si]
            assert 0 <= so and so + nb <= s.size, "source range out of bounds"
            d[do:do + nb] = s[so:so + nb]


@pytest.mark.parametrize("chunk", [4096, 65536])
@pytest.mark.parametrize("sizes,G,esz", LAYOUTS)
def test_copy_plans_reproduce_oracle(sizes, G, esz, chunk):
    dt = np.uint16 if esz == 2 else np.uint32
    tr = [(t * 5 + G) % 2 == 0 for t in range(len(sizes))]
    old = fcdp.fcdp_tuning_get("copy_chunk_bytes")
    fcdp.fcdp_tuning_set("copy_chunk_bytes", chunk)
    try:
        L = fcdp.fcdp_layout_build(sizes, tr, G, esz)
    finally:
        fcdp.fcdp_tuning_set("copy_chunk_bytes", old)
    tensors = _rand_tensors(len(sizes), sizes, dt)
    flat = oracle.flatten(tensors, G)
    shards = oracle.split(flat, G)
    sb = [s.view(np.uint8) for s in shards]
    # unflatten
    plan = L.copy_plan(0)
    assert all(nb <= chunk for *_x, nb in plan)
    out = [np.full(k * esz, 0xEE, np.uint8) for k in sizes]
    _run_plan(plan, sb, out)
    for t, w in enumerate(oracle.materialize_from_shards(shards, sizes) if L.shard_numel else tensors):
        assert np.array_equal(out[t].view(dt), w)
    assert sum(nb for *_x, nb in plan) == L.numel * esz
    # flatten (with zero tail)
    back = [np.full(L.shard_numel * esz, 0xEE, np.uint8) for _ in range(G)]
    _run_plan(L.copy_plan(1), [t.view(np.uint8) for t in tensors], back)
    for r in range(G):
        assert np.array_equal(back[r].view(dt), shards[r])
    # pack / unpack
    packed = [np.full(L.packed_numel * esz, 0xEE, np.uint8)]
    _run_plan(L.copy_plan(2), [flat.view(np.uint8)], packed)
    assert np.array_equal(packed[0].view(dt), oracle.pack(flat, sizes, tr, G))
    base = _rand_tensors(77, [flat.size], dt)[0]
    want = base.copy()
    oracle.unpack(packed[0].view(dt), want, sizes, tr)
    got = [base.copy().view(np.uint8)]
    _run_plan(L.copy_plan(3), packed, got)
    assert np.array_equal(got[0].view(dt), want)


def _covered_exactly_once(plan, dst_sizes):
    """Every destination byte is written by exactly one row of the plan."""
    cover = [np.zeros(n, dtype=np.uint8) for n in dst_sizes]
    for _si, _so, di, do, nb in plan:
        cover[di][do:do + nb] += 1
    return all(bool(np.all(c == 1)) for c in cover)


@settings(max_examples=60, deadline=None, derandomize=True)
@given(sizes=st.lists(st.one_of(st.integers(0, 3), st.integers(0, 40000),
                                st.sampled_from([2048, 4096, 8192, 32768, 2047, 4097])),
                      min_size=1, max_size=12),
       G=st.sampled_from([1, 2, 3, 4, 5, 7, 8, 16, 32, 64]),
       esz=st.sampled_from([2, 4]), chunk=st.sampled_from([4096, 8192, 65536]))
def test_copy_plans_property(sizes, G, esz, chunk):
    """Random layouts: the plans are in bounds, write every destination byte
    exactly once and reproduce the oracle (same checks as above)."""
    test_copy_plans_reproduce_oracle(sizes, G, esz, chunk)
    tr = [(t * 5 + G) % 2 == 0 for t in range(len(sizes))]
    old = fcdp.fcdp_tuning_get("copy_chunk_bytes")
    fcdp.fcdp_tuning_set("copy_chunk_bytes", chunk)
    try:
        L = fcdp.fcdp_layout_build(sizes, tr, G, esz)
    finally:
        fcdp.fcdp_tuning_set("copy_chunk_bytes", old)
    assert _covered_exactly_once(L.copy_plan(0), [k * esz for k in sizes])
    assert _covered_exactly_once(L.copy_plan(1), [L.shard_numel * esz] * G)
    assert _covered_exactly_once(L.copy_plan(2), [L.packed_numel * esz])
    # unpack writes exactly the trainable ranges of the flat buffer
    cover = np.zeros(L.padded_numel * esz, dtype=np.uint8)
    for _si, _so, _di, do, nb in L.copy_plan(3):
        cover[do:do + nb] += 1
    want = np.zeros_like(cover)
    for t, k in enumerate(sizes):
        if tr[t]:
            want[L.offsets[t] * esz:(L.offsets[t] + k) * esz] = 1
    assert np.array_equal(cover, want)


def test_copy_plan_at_benchmark_shapes():
    """Plans of the five benchmark shapes: in bounds, cover N exactly, cuts on
    16-byte boundaries (these shapes never need the scalar head/tail path)."""
    for name, cfg in synth.CONFIGS.items():
        L = fcdp.fcdp_layout_build(cfg.numel, cfg.trainable, cfg.G, 2)
        plan = np.array(L.copy_plan(0), dtype=np.int64).reshape(-1, 5)
        assert int(plan[:, 4].sum()) == cfg.N * 2
        assert np.all(plan[:, 1] % 16 == 0) and np.all(plan[:, 3] % 16 == 0)
        assert np.all(plan[:, 4] % 16 == 0)
        S2 = L.shard_numel * 2
        assert np.all(plan[:, 1] + plan[:, 4] <= S2)
        numel = np.array(cfg.numel)
        assert np.all(plan[:, 3] + plan[:, 4] <= numel[plan[:, 2]] * 2)
        assert plan[:, 0].min() >= 0 and plan[:, 0].max() < cfg.G


def test_huge_layer_plans_stay_bounded():
    """A 16 GiB layer (beyond any shipped shape): the piece size grows so that
    no table exceeds about 4 M pieces, offsets stay 64-bit clean, and the plan
    still covers every byte exactly (checked by sums and by order, without
    allocating the layer)."""
    sizes = [2 ** 32, 2 ** 32 + 12345, 7, 2 ** 31 + 1]
    G = 64
    L = fcdp.fcdp_layout_build(sizes, [0, 1, 1, 0], G, 2)
    lay = oracle.layout(sizes, G)
    assert (L.numel, L.padded_numel, L.shard_numel) == (lay["N"], lay["N_pad"], lay["S"])
    lib = fcdp.load_library()
    for which, total in ((0, L.numel * 2), (1, L.padded_numel * 2),
                         (2, L.packed_numel * 2), (3, L.trainable_numel * 2)):
        n = lib.fcdp_layout_copy_plan(L.handle, which, None, 0)
        assert 0 < n <= (1 << 22) + 4 * (len(sizes) + G)
        rows = np.zeros((n, 5), dtype=np.int64)
        assert lib.fcdp_layout_copy_plan(L.handle, which, ctypes.c_void_p(rows.ctypes.data), n) == n
        assert int(rows[:, 4].sum()) == total
        assert rows[:, 4].min() > 0 and np.all(rows[:, 4] % 2 == 0)
        assert rows[:, 1].min() >= 0 and rows[:, 3].min() >= 0
        # destination ranges of one buffer follow each other without gap or overlap
        for di in np.unique(rows[:, 2])[:3]:
            r = rows[rows[:, 2] == di]
            r = r[np.argsort(r[:, 3], kind="stable")]
            assert np.all(r[1:, 3] == r[:-1, 3] + r[:-1, 4])
    segs = np.array(L.segments(), dtype=np.int64).reshape(-1, 5)
    assert np.array_equal(segs, oracle.segments(sizes, G))


def test_layout_build_errors():
    E = fcdp.FcdpError
    for args, name in [
        (([1, 2], None, 0), "FCDP_EINVAL"),
        (([1, 2], None, 65), "FCDP_ESIZE"),
        (([1, -2], None, 2), "FCDP_EINVAL"),
        (([], None, 2), "FCDP_EINVAL"),
        (([2 ** 61, 2 ** 61], None, 2), "FCDP_ESIZE"),
    ]:
        with pytest.raises(E) as e:
            fcdp.fcdp_layout_build(*args)
        assert e.value.name == name, args
    with pytest.raises(E):
        fcdp.fcdp_layout_build([4], None, 2, 3)
    with pytest.raises(E):
        fcdp.fcdp_layout_build([4], None, 2, 2, 0)
    lib = fcdp.load_library()
    assert lib.fcdp_layout_build(None, None, 1, 1, 2, 64, None) == 1
    out = ctypes.c_void_p()
    assert lib.fcdp_layout_build(None, None, 1, 1, 2, 64, ctypes.byref(out)) == 1
    assert b"numel" in lib.fcdp_last_error()
    assert lib.fcdp_layout_numel(None) == -1
    lib.fcdp_layout_destroy(None)


def test_data_call_argument_errors_before_any_enqueue():
    """These fail on argument checks alone, so they need no GPU."""
    E = fcdp.FcdpError
    L = fcdp.fcdp_layout_build([1000, 24], None, 4, 2)
    good = [0x1000, 0x2000]
    sh = [0x10000 * (r + 1) for r in range(4)]

    def err(fn, *a):
        with pytest.raises(E) as e:
            fn(*a)
        return e.value.name

    m = fcdp.fcdp_materialize_layer
    assert err(m, L, 9, sh, None, None, good) == "FCDP_EINVAL"
    assert err(m, L, fcdp.SRC_DEVICE_SHARDS, None, None, None, good) == "FCDP_EINVAL"
    assert err(m, L, fcdp.SRC_DEVICE_SHARDS, sh, None, None, None) == "FCDP_EINVAL"
    assert err(m, L, fcdp.SRC_DEVICE_SHARDS, sh, None, None, [0x1002, 0x2000]) == "FCDP_EALIGN"
    assert err(m, L, fcdp.SRC_DEVICE_SHARDS, [0x10, 0x20, 0x30, 0x38], None, None, good) == "FCDP_EALIGN"
    assert err(m, L, fcdp.SRC_DEVICE_SHARDS, [0x10, 0x20, 0, 0x40], None, None, good) == "FCDP_EINVAL"
    assert err(m, L, fcdp.SRC_DEVICE_SHARDS, sh, None, None, good, True) == "FCDP_EINVAL"
    assert err(m, L, fcdp.SRC_HOST_DMA, None, 0x5000, None, good) == "FCDP_EINVAL"
    assert err(m, L, fcdp.SRC_HOST_DMA, None, None, 0x6000, good) == "FCDP_EINVAL"
    assert err(m, L, fcdp.SRC_HOST_DMA, None, 0x5004, 0x6000, good) == "FCDP_EALIGN"
    assert err(m, L, fcdp.SRC_HOST_DMA, None, 0x5000, 0x6000, good, True) == "FCDP_EINVAL"
    assert err(m, L, fcdp.SRC_HOST_ZEROCOPY, None, None, None, good) == "FCDP_EINVAL"
    r = fcdp.fcdp_reduce_grad_shard
    assert err(r, None, 2, 0, 10, fcdp.F32, fcdp.F32, 0x9000) == "FCDP_EINVAL"
    assert err(r, [0x100, 0x200], 0, 0, 10, fcdp.F32, fcdp.F32, 0x9000) == "FCDP_EINVAL"
    assert err(r, [0x100] * 65, 65, 0, 10, fcdp.F32, fcdp.F32, 0x9000) == "FCDP_ESIZE"
    assert err(r, [0x100, 0x200], 2, 0, -1, fcdp.F32, fcdp.F32, 0x9000) == "FCDP_EINVAL"
    assert err(r, [0x100, 0x200], 2, -1, 10, fcdp.F32, fcdp.F32, 0x9000) == "FCDP_EINVAL"
    assert err(r, [0x100, 0x200], 2, 0, 10, 5, fcdp.F32, 0x9000) == "FCDP_EINVAL"
    assert err(r, [0x100, 0x200], 2, 0, 10, fcdp.F32, fcdp.F32, None) == "FCDP_EINVAL"
    assert err(r, [0x100, 0x204], 2, 0, 10, fcdp.F32, fcdp.F32, 0x9000) == "FCDP_EALIGN"
    assert err(r, [0x100, 0x200], 2, 0, 10, fcdp.F32, fcdp.F32, 0x9008) == "FCDP_EALIGN"
    assert err(r, [0x100, 0], 2, 0, 10, fcdp.F32, fcdp.F32, 0x9000) == "FCDP_EINVAL"
    # partial overlap of output and an input; exact in-place with a narrower output dtype
    assert err(r, [0x1000, 0x8000], 2, 0, 100, fcdp.F32, fcdp.F32, 0x1010) == "FCDP_EINVAL"
    assert err(r, [0x1000, 0x8000], 2, 0, 100, fcdp.F32, fcdp.BF16, 0x1000) == "FCDP_EINVAL"
    rs = fcdp.fcdp_reduce_grad_shard_scaled
    assert err(rs, [0x100, 0x200], 2, 0, 10, fcdp.F32, fcdp.F32, float("nan"), 0x9000) == "FCDP_EINVAL"
    assert err(rs, [0x100, 0x200], 2, 0, 10, fcdp.F32, fcdp.F32, float("inf"), 0x9000) == "FCDP_EINVAL"
    assert err(rs, [0x100, 0x204], 2, 0, 10, fcdp.F32, fcdp.F32, 0.5, 0x9000) == "FCDP_EALIGN"
    assert err(fcdp.fcdp_reduce_trainable_shard_scaled, L, [0x100000, 0x200000, 0x300000, 0x400000],
               0, fcdp.F32, fcdp.F32, float("-inf"), 0x9000) == "FCDP_EINVAL"
    p = fcdp.fcdp_pack_trainable
    assert err(p, L, None, 0x100) == "FCDP_EINVAL"
    assert err(p, L, 0x104, 0x10000) == "FCDP_EALIGN"
    assert err(p, L, 0x1000, 0x1100) == "FCDP_EINVAL"       # overlap
    assert err(fcdp.fcdp_unpack_trainable, L, 0x1000, 0x1100) == "FCDP_EINVAL"
    assert err(fcdp.fcdp_flatten_to_shards, L, None, sh) == "FCDP_EINVAL"
    assert err(fcdp.fcdp_probe_copy, 0x1000, 0x2001, 64) == "FCDP_EALIGN"
    assert err(fcdp.fcdp_tuning_set, "no_such_knob", 1) == "FCDP_EINVAL"
    assert err(fcdp.fcdp_tuning_set, "copy_block", 100) == "FCDP_EINVAL"
    assert fcdp.fcdp_tuning_get("no_such_knob") == -1
    lib = fcdp.load_library()
    out = ctypes.c_void_p()
    assert lib.fcdp_host_cache_alloc(0, -1, ctypes.byref(out), ctypes.byref(out)) == 1
    assert lib.fcdp_host_cache_alloc(16, -1, None, None) == 1


def test_empty_layer_is_a_no_op():
    L = fcdp.fcdp_layout_build([0, 0, 0], None, 4, 2)
    assert (L.numel, L.padded_numel, L.shard_numel, L.packed_numel) == (0, 0, 0, 0)
    sh = [0x100 * (r + 1) for r in range(4)]
    fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, sh, None, None, [None, None, None])
    fcdp.fcdp_flatten_to_shards(L, [None] * 3, sh)
    fcdp.fcdp_pack_trainable(L, 0x1000, 0x2000)
    fcdp.fcdp_unpack_trainable(L, 0x2000, 0x1000)
    fcdp.fcdp_reduce_grad_shard([0x100, 0x200], 2, 0, 0, fcdp.F32, fcdp.F32, 0x9000)


def _drive_state(layers, iterations, host_mode):
    """Runs the library's dirty flags through the loop of Alg. 1."""
    st = fcdp.CacheState(len(layers))
    events = []
    for it in range(iterations):
        for l, layer in enumerate(layers):
            classes = sorted(set(int(tr) for _n, _k, tr in layer))
            dec = {}
            for c in classes:
                dec[c] = st.forward_source(l, c, host_mode)
            for name, _k, tr in layer:
                src, store = dec[int(tr)]
                if src == fcdp.SRC_DEVICE_SHARDS:
                    assert store
                    events.append((it, "fwd", l, name, alg1.INTER))
                    events.append((it, "fwd", l, name, "store"))
                else:
                    assert src == host_mode and not store
                    events.append((it, "fwd", l, name, alg1.HOST))
        for l in range(len(layers) - 1, -1, -1):
            for name, _k, tr in layers[l]:
                assert st.backward_source(l, int(tr), host_mode) == host_mode
                events.append((it, "bwd", l, name, alg1.HOST))
        events.append((it, "rs", -1, "grad_W_t", alg1.INTER))
        st.optimizer_step()
        for l, layer in enumerate(layers):
            for name, _k, tr in layer:
                if tr:
                    events.append((it, "upd", l, name, "dirty"))
    return st, events


@pytest.mark.parametrize("peft", [False, True])
def test_cache_state_follows_alg1(peft):
    if peft:
        layers = [[("base", 1000, False), ("lora_A", 10, True), ("lora_B", 10, True)] for _ in range(5)]
    else:
        layers = [[("w", 1000, True), ("b", 10, True)] for _ in range(5)]
    st, events = _drive_state(layers, 4, fcdp.SRC_HOST_DMA)
    want = alg1.replay(layers, 4)
    assert events == want["events"]
    for l in range(5):
        assert st.is_dirty(l, 1) == 1
        assert st.is_dirty(l, 0) == (0 if peft else 1)   # class 0 unused when all trainable


def test_cache_state_errors():
    st = fcdp.CacheState(2)
    with pytest.raises(fcdp.FcdpError) as e:
        st.backward_source(0, 0, fcdp.SRC_HOST_DMA)     # nothing stored yet
    assert e.value.name == "FCDP_ESTATE"
    with pytest.raises(fcdp.FcdpError):
        st.forward_source(2, 0, fcdp.SRC_HOST_DMA)
    with pytest.raises(fcdp.FcdpError):
        st.forward_source(0, 2, fcdp.SRC_HOST_DMA)
    with pytest.raises(fcdp.FcdpError):
        st.forward_source(0, 0, fcdp.SRC_DEVICE_SHARDS)
    assert st.is_dirty(5, 0) == -1
    with pytest.raises(fcdp.FcdpError):
        fcdp.CacheState(0)


def test_failed_store_can_be_rolled_back():
    """forward_source marks a class clean before the caller's store runs; if
    the store fails the caller marks it dirty again: backward_source refuses
    to serve an image that was never written, and the next forward pass is a
    miss again."""
    st = fcdp.CacheState(3)
    assert st.forward_source(1, 0, fcdp.SRC_HOST_DMA) == (fcdp.SRC_DEVICE_SHARDS, True)
    assert st.is_dirty(1, 0) == 0
    assert st.backward_source(1, 0, fcdp.SRC_HOST_DMA) == fcdp.SRC_HOST_DMA   # would serve it
    st.mark_dirty(1, 0)                                                      # ... the store failed
    assert st.is_dirty(1, 0) == 1
    with pytest.raises(fcdp.FcdpError) as e:
        st.backward_source(1, 0, fcdp.SRC_HOST_DMA)
    assert e.value.name == "FCDP_ESTATE"
    assert st.forward_source(1, 0, fcdp.SRC_HOST_DMA) == (fcdp.SRC_DEVICE_SHARDS, True)
    # a resident layer loses its residency too
    st.set_tau(1.0)
    st.forward_source(2, 1, fcdp.SRC_HOST_DMA)
    assert st.place(2, 1, 100) is True
    assert st.backward_source(2, 1, fcdp.SRC_HOST_DMA) == fcdp.SRC_DEVICE_RESIDENT
    st.mark_dirty(2, 1)
    with pytest.raises(fcdp.FcdpError):
        st.backward_source(2, 1, fcdp.SRC_HOST_DMA)
    for bad in ((3, 0), (-1, 0), (0, 2)):
        with pytest.raises(fcdp.FcdpError) as e:
            st.mark_dirty(*bad)
        assert e.value.name == "FCDP_EINVAL"


def test_no_gpu_means_loud_failure():
    """Without a device a valid data call returns FCDP_EHIP; it never falls
    back to a CPU path."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    L = fcdp.fcdp_layout_build([1024], None, 2, 2)
    with pytest.raises(fcdp.FcdpError) as e:
        fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, [0x1000, 0x2000], None, None, [0x8000])
    assert e.value.name in ("FCDP_EHIP", "FCDP_ENOMEM")


def test_adaptive_placement_follows_the_oracle():
    """The library's keep/offload decisions, residency and dirty flags against
    the Sec. 4.4 replay (full fine-tuning, utilisation rising with depth)."""
    nl = 6
    sizes = [1000 + 10 * l for l in range(nl)]

    def util(it, l):
        return min(0.95, 0.25 + 0.1 * l + 0.05 * it)

    for tau in (0.0, 0.4, 0.62, 1.0):
        st = fcdp.CacheState(nl)
        st.set_tau(tau)
        want = alg1.replay_adaptive(sizes, util, tau, 3)["iterations"]
        for it in range(3):
            kept, stored, fetched = [], 0, 0
            for l in range(nl):
                src, store = st.forward_source(l, 1, fcdp.SRC_HOST_DMA)
                assert src == fcdp.SRC_DEVICE_SHARDS and store      # every forward is a miss
                total = 1 << 30
                if st.place(l, int(util(it, l) * total), total):
                    kept.append(l)
                    assert st.is_dirty(l, 1) == 1       # the host copy was not refreshed
                else:
                    stored += sizes[l]
                    assert st.is_dirty(l, 1) == 0
            for l in range(nl - 1, -1, -1):
                src = st.backward_source(l, 1, fcdp.SRC_HOST_DMA)
                if l in kept:
                    assert src == fcdp.SRC_DEVICE_RESIDENT
                else:
                    assert src == fcdp.SRC_HOST_DMA
                    fetched += sizes[l]
                st.release(l)
            assert {"kept": kept, "stored": stored, "fetched": fetched} == want[it]
            st.optimizer_step()
    st = fcdp.CacheState(2)
    with pytest.raises(fcdp.FcdpError):
        st.set_tau(1.5)
    with pytest.raises(fcdp.FcdpError):
        st.place(0, 10, 0)
    with pytest.raises(fcdp.FcdpError):
        st.place(5, 1, 10)
    # a released layer that was never stored cannot be served in a backward pass
    st.set_tau(1.0)
    st.forward_source(0, 1, fcdp.SRC_HOST_DMA)
    assert st.place(0, 1, 10)
    st.release(0)
    with pytest.raises(fcdp.FcdpError) as e:
        st.backward_source(0, 1, fcdp.SRC_HOST_DMA)
    assert e.value.name == "FCDP_ESTATE"
