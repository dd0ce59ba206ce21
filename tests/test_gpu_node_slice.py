"""One GPU's share of a node (Sec. 4.3, backward pass: each GPU loads its 1/g
part of the cached layer from host memory, the node's GPUs exchange the
parts): the slice store and the slice fetch against the oracle.

The oracle needs no new arithmetic: the slice store must leave the bytes of
concat(own shards) in the host slice, and the fetch, given the host slice and
the peers' shards on the device, must give what materialize_from_shards gives
for all G shards."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_06499_amd as fcdp
from paper_2602_06499_amd import synth
from gpu_util import Arena

pytestmark = pytest.mark.gpu


def _rand_tensors(seed, sizes, dtype):
    g = synth.rng(0, seed, synth.KIND_MISC, 23)
    info = np.iinfo(dtype)
    return [g.integers(0, int(info.max) + 1, size=k, dtype=dtype) for k in sizes]


CASES = [  # G, GPUs per node g, element size, tensors, largest tensor
    (4, 2, 2, 9, 70000), (8, 8, 2, 12, 300000), (8, 2, 4, 5, 50000), (16, 4, 2, 20, 90000),
    (32, 8, 2, 7, 400000), (6, 3, 2, 4, 33333), (64, 8, 2, 30, 20000), (4, 4, 2, 3, 100),
    (8, 1, 2, 6, 65536),      # g = 1: the slice is the whole layer
]


@pytest.mark.parametrize("G,g,esz,T,max_numel", CASES)
def test_node_slice_store_and_fetch(G, g, esz, T, max_numel):
    dt = np.uint16 if esz == 2 else np.uint32
    sizes = synth.random_layer(7000 + G * 10 + g, T=T, max_numel=max_numel)
    tensors = _rand_tensors(G * 100 + g, sizes, dt)
    flat = oracle.flatten(tensors, G)
    shards = oracle.split(flat, G)
    want = oracle.materialize_from_shards(shards, sizes)
    image = oracle.cache_store(shards)
    L = fcdp.fcdp_layout_build(sizes, None, G, esz)
    L.prepare()
    S = L.shard_numel
    n = G // g
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    sh = Arena([S * esz] * G)                       # G separate shard buffers
    for r in range(G):
        sh.fill(r, shards[r])
    for k in range(g):                              # every GPU of the node in turn
        first = k * n
        H = fcdp.fcdp_host_cache_alloc(n * S * esz + 64)
        H.numpy(np.uint8)[:] = 0x5A
        # ---- store: only the slice's shard pointers are read
        ptrs = [sh.ptr(r) if first <= r < first + n else None for r in range(G)]
        fcdp.fcdp_link_bytes(True)
        fcdp.fcdp_cache_store_node_slice(L, first, n, ptrs, H, compute, copy)
        torch.cuda.synchronize()
        assert np.array_equal(H.numpy(dt, n * S), image[first * S:(first + n) * S]), (k, "store")
        assert np.all(H.numpy(np.uint8)[n * S * esz:] == 0x5A), "the store wrote past the slice"
        assert fcdp.fcdp_link_bytes()[0] == n * S * esz
        # ---- fetch: the slice from the host, every other shard from the device; the
        # slice's own device pointers are not passed at all
        peers = [None if first <= r < first + n else sh.ptr(r) for r in range(G)]
        staging = Arena([n * S * esz])
        out = Arena([kk * esz for kk in sizes])
        fcdp.fcdp_link_bytes(True)
        fcdp.fcdp_materialize_layer_node_slice(L, first, n, peers, H, staging.ptr(0), out.ptrs(), compute, copy)
        torch.cuda.synchronize()
        for t in range(len(sizes)):
            assert np.array_equal(out.get(t, dt), want[t]), (k, "fetch", t)
        out.check_guards()
        staging.check_guards()
        assert fcdp.fcdp_link_bytes()[1] == n * S * esz
        H.free()
    sh.check_guards()


def test_node_slice_full_size_70b_share():
    """One Llama-70B-shaped layer, G = 32, a node of 8 GPUs: GPU 3's share is
    shards 12..15 (214 MB of the 1.7 GB layer); store, fetch, compare."""
    cfg = synth.CONFIGS["llama70b_g32"]
    G, g, k = cfg.G, 8, 3
    n, first = G // g, 3 * (G // g)
    dev = torch.device("cuda:0")
    L = fcdp.fcdp_layout_build(cfg.numel, cfg.trainable, G, 2)
    L.prepare()
    Np, S = L.padded_numel, L.shard_numel
    gen = synth.torch_device_generator(dev, cfg.config_id, 5, synth.KIND_PARAM)
    gathered = torch.empty(Np, dtype=torch.bfloat16, device=dev).normal_(0.0, 0.02, generator=gen)
    off = L.offsets
    H = fcdp.fcdp_host_cache_alloc(n * S * 2)
    staging = torch.empty(n * S, dtype=torch.bfloat16, device=dev)
    tensors = [torch.zeros(max(kk, 1), dtype=torch.bfloat16, device=dev) for kk in cfg.numel]
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    all_ptrs = [gathered.data_ptr() + r * S * 2 for r in range(G)]
    torch.cuda.synchronize()
    fcdp.fcdp_cache_store_node_slice(L, first, n, all_ptrs, H, compute, copy)
    torch.cuda.synchronize()
    hs = torch.from_numpy(H.numpy(np.int16, n * S))
    assert torch.equal(hs, gathered[first * S:(first + n) * S].cpu().view(torch.int16))
    # the peers' shards on the device, this GPU's own range overwritten so that only the host copy can be right
    scratch = gathered.clone()
    scratch[first * S:(first + n) * S] = 0
    peers = [None if first <= r < first + n else scratch.data_ptr() + r * S * 2 for r in range(G)]
    torch.cuda.synchronize()
    fcdp.fcdp_materialize_layer_node_slice(L, first, n, peers, H, staging, tensors, compute, copy)
    torch.cuda.synchronize()
    for t, kk in enumerate(cfg.numel):
        assert torch.equal(tensors[t][:kk], gathered[off[t]:off[t] + kk]), t
    # and against the oracle's definition on all G shards
    flat = gathered.cpu().view(torch.int16).numpy().view(np.uint16)
    want = oracle.materialize_from_shards([flat[r * S:(r + 1) * S] for r in range(G)], list(cfg.numel))
    for t, kk in enumerate(cfg.numel):
        assert np.array_equal(tensors[t][:kk].cpu().view(torch.int16).numpy().view(np.uint16), want[t]), t
    H.free()


def test_node_slice_arguments():
    sizes, G = [4096, 100, 7000], 4
    L = fcdp.fcdp_layout_build(sizes, None, G, 2)
    L.prepare()
    S = L.shard_numel
    sh = Arena([S * 2] * G)
    out = Arena([k * 2 for k in sizes])
    staging = Arena([2 * S * 2])
    H = fcdp.fcdp_host_cache_alloc(2 * S * 2)
    for first, n in ((-1, 2), (3, 2), (0, 0), (0, 5), (4, 1)):
        for call in (lambda: fcdp.fcdp_cache_store_node_slice(L, first, n, sh.ptrs(), H),
                     lambda: fcdp.fcdp_materialize_layer_node_slice(L, first, n, sh.ptrs(), H, staging.ptr(0), out.ptrs())):
            with pytest.raises(fcdp.FcdpError) as e:
                call()
            assert e.value.name == "FCDP_EINVAL", (first, n)
    peers = sh.ptrs()
    peers[0] = None                                 # a peer's shard is missing
    with pytest.raises(fcdp.FcdpError) as e:
        fcdp.fcdp_materialize_layer_node_slice(L, 1, 2, peers, H, staging.ptr(0), out.ptrs())
    assert e.value.name == "FCDP_EINVAL"
    with pytest.raises(fcdp.FcdpError) as e:
        fcdp.fcdp_materialize_layer_node_slice(L, 1, 2, sh.ptrs(), H, None, out.ptrs())
    assert e.value.name == "FCDP_EINVAL"
    with pytest.raises(fcdp.FcdpError) as e:
        fcdp.fcdp_materialize_layer_node_slice(L, 1, 2, sh.ptrs(), H.host + 2, staging.ptr(0), out.ptrs())
    assert e.value.name == "FCDP_EALIGN"
    own = [None, sh.ptr(1), sh.ptr(2), None]         # the store reads the slice's pointers only
    fcdp.fcdp_cache_store_node_slice(L, 1, 2, own, H)
    own[2] = None
    with pytest.raises(fcdp.FcdpError) as e:
        fcdp.fcdp_cache_store_node_slice(L, 1, 2, own, H)
    assert e.value.name == "FCDP_EINVAL"
    torch.cuda.synchronize()
    out.check_guards()
    H.free()


def test_node_slice_backward_sweep_two_staging_slices():
    """Eight layers fetched back to back through two alternating staging
    slices with the copy stream held back at the start: every layer's tensors
    are its own (the staging bookkeeping orders copy(l+2) after scatter(l))."""
    sizes, G, g = [300000, 7, 65536, 123457], 8, 4
    n, first = G // g, 2
    L = fcdp.fcdp_layout_build(sizes, None, G, 2)
    L.prepare()
    S = L.shard_numel
    nl = 8
    layers = [_rand_tensors(600 + l, sizes, np.uint16) for l in range(nl)]
    shards = [oracle.split(oracle.flatten(layers[l], G), G) for l in range(nl)]
    H = fcdp.fcdp_host_cache_alloc(nl * n * S * 2)
    for l in range(nl):
        H.numpy(np.uint16, n * S, l * n * S * 2)[:] = np.concatenate(shards[l][first:first + n])
    dev_sh = [Arena([S * 2] * G) for _ in range(nl)]
    for l in range(nl):
        for r in range(G):
            if not first <= r < first + n:
                dev_sh[l].fill(r, shards[l][r])
    outs = [Arena([k * 2 for k in sizes]) for _ in range(nl)]
    stg = Arena([n * S * 2, n * S * 2])
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(copy):
        torch.cuda._sleep(50_000_000)
    for l in range(nl - 1, -1, -1):
        peers = [None if first <= r < first + n else dev_sh[l].ptr(r) for r in range(G)]
        fcdp.fcdp_materialize_layer_node_slice(L, first, n, peers, H.host + l * n * S * 2, stg.ptr(l % 2),
                                               outs[l].ptrs(), compute, copy)
    torch.cuda.synchronize()
    for l in range(nl):
        want = oracle.materialize_from_shards(shards[l], sizes)
        for t in range(len(sizes)):
            assert np.array_equal(outs[l].get(t, np.uint16), want[t]), (l, t)
        outs[l].check_guards()
    stg.check_guards()
    H.free()


def test_node_slice_training_loop_stays_coherent():
    """Full fine-tuning over three iterations as GPU 1 of a node of 2 (Alg. 1's
    flags decide: every forward is a miss, because the step dirtied the layer,
    and refreshes this GPU's host slice; every backward is a hit and takes the
    slice from the host and the other half from the peer's shards): the
    tensors of both passes are the current parameters, never last step's."""
    sizes, G, g, k = [50000, 3, 131072, 70001], 8, 2, 1
    n, first = G // g, k * (G // g)
    nl, iters = 3, 3
    L = fcdp.fcdp_layout_build(sizes, None, G, 2)
    L.prepare()
    S = L.shard_numel
    rng = synth.rng(0, 808, synth.KIND_MISC)
    params = [[rng.integers(0, 65536, size=kk, dtype=np.uint16) for kk in sizes] for _ in range(nl)]
    H = fcdp.fcdp_host_cache_alloc(nl * n * S * 2)
    H.numpy(np.uint16)[:] = 0xDEAD
    state = fcdp.CacheState(nl)
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    stg = Arena([n * S * 2, n * S * 2])
    for it in range(iters):
        gathered = []
        for l in range(nl):                                   # ---- forward
            src, store = state.forward_source(l, 1, fcdp.SRC_HOST_DMA)
            assert (src, store) == (fcdp.SRC_DEVICE_SHARDS, True)
            shards = oracle.split(oracle.flatten(params[l], G), G)
            sh = Arena([S * 2] * G)                           # what the inter-node gather delivered
            for r in range(G):
                sh.fill(r, shards[r])
            gathered.append((sh, shards))
            out = Arena([kk * 2 for kk in sizes])
            fcdp.fcdp_materialize_layer(L, src, sh.ptrs(), None, None, out.ptrs(), fcdp.STORE_NONE, compute, copy)
            fcdp.fcdp_cache_store_node_slice(L, first, n, sh.ptrs(), H.host + l * n * S * 2, compute, copy)
            torch.cuda.synchronize()
            for t in range(len(sizes)):
                assert np.array_equal(out.get(t, np.uint16), params[l][t]), ("forward", it, l, t)
        for l in range(nl - 1, -1, -1):                       # ---- backward
            assert state.backward_source(l, 1, fcdp.SRC_HOST_DMA) == fcdp.SRC_HOST_DMA
            sh, shards = gathered[l]
            # after the forward pass only the peer's half is back on this GPU (the exchange inside
            # the node); this GPU's own half of the gathered buffer was freed: overwrite it
            for r in range(first, first + n):
                sh.fill(r, np.full(S, 0xBEEF, dtype=np.uint16))
            peers = [None if first <= r < first + n else sh.ptr(r) for r in range(G)]
            out = Arena([kk * 2 for kk in sizes])
            fcdp.fcdp_materialize_layer_node_slice(L, first, n, peers, H.host + l * n * S * 2, stg.ptr(l % 2),
                                                   out.ptrs(), compute, copy)
            torch.cuda.synchronize()
            for t in range(len(sizes)):
                assert np.array_equal(out.get(t, np.uint16), params[l][t]), ("backward", it, l, t)
            out.check_guards()
        for l in range(nl):                                   # ---- the optimizer changes every parameter
            params[l] = [(p + np.uint16(it * 7 + l + 1)).astype(np.uint16) for p in params[l]]
        state.optimizer_step()
    stg.check_guards()
    H.free()


UNPACK_CASES = [  # G, g, element size, tensors, largest tensor
    (4, 2, 2, 9, 70000), (8, 4, 2, 14, 30000), (8, 8, 4, 6, 50000), (16, 2, 2, 25, 9000),
    (6, 3, 2, 5, 33333), (32, 8, 2, 40, 20000), (4, 4, 2, 3, 50),
]


@pytest.mark.parametrize("G,g,esz,T,max_numel", UNPACK_CASES)
def test_unpack_into_a_node_slice(G, g, esz, T, max_numel):
    """Unpack restricted to a GPU's shards: the slice ends up as the same
    range of the flat image the oracle's unpack produces; frozen bytes of the
    slice and everything around it stay as they were."""
    dt = np.uint16 if esz == 2 else np.uint32
    sizes = synth.random_layer(8100 + G * 10 + g, T=T, max_numel=max_numel)
    rng = synth.rng(0, 8200 + G + g, synth.KIND_MISC)
    tr = [int(v) for v in rng.integers(0, 2, size=T)]
    if g == 4 and G == 4:
        tr = [0] * T                                # no trainable tensor at all: a no-op
    tensors = _rand_tensors(G * 100 + g + 7, sizes, dt)
    flat = oracle.flatten(tensors, G)
    L = fcdp.fcdp_layout_build(sizes, tr, G, esz)
    L.prepare()
    S, Pn = L.shard_numel, L.packed_numel
    info = np.iinfo(dt)
    packed = rng.integers(0, int(info.max) + 1, size=Pn, dtype=dt)
    want_flat = flat.copy()
    oracle.unpack(packed, want_flat, sizes, tr)
    d_packed = Arena([max(Pn * esz, 16)])
    if Pn:
        d_packed.fill(0, packed)
    n = G // g
    st = torch.cuda.Stream()
    for k in range(g):
        first = k * n
        sl = Arena([max(n * S * esz, 16)])
        if n * S:
            sl.fill(0, flat[first * S:(first + n) * S])   # the slice before the refresh
        torch.cuda.synchronize()
        fcdp.fcdp_unpack_trainable_node_slice(L, first, n, d_packed.ptr(0), sl.ptr(0), st)
        torch.cuda.synchronize()
        if n * S:
            assert np.array_equal(sl.get(0, dt), want_flat[first * S:(first + n) * S]), (k, "slice")
        sl.check_guards()
    d_packed.check_guards()
    if any(tr) and L.trainable_numel:
        # the slices together changed exactly what the whole-buffer unpack changes
        assert not np.array_equal(want_flat, flat) or np.array_equal(packed[:L.trainable_numel],
                                                                    oracle.pack(flat, sizes, tr, G)[:L.trainable_numel])


def test_peft_loop_through_node_slices():
    """Alg. 1 under PEFT as GPU 0 of a node of 2, three iterations: the first
    forward is a miss (store this GPU's slice); later forwards hit for the
    frozen class and refresh the trainable ranges of this GPU's host slice by
    the clipped unpack through the mapping; every backward takes the slice
    from the host.  The tensors are always the current parameters."""
    sizes, G, g, k = [40000, 4096, 77777, 512, 90001], 4, 2, 0
    trainable = [0, 1, 0, 1, 0]
    n, first = G // g, k * (G // g)
    nl, iters = 2, 3
    L = fcdp.fcdp_layout_build(sizes, trainable, G, 2)
    L.prepare()
    S = L.shard_numel
    rng = synth.rng(0, 909, synth.KIND_MISC)
    params = [[rng.integers(0, 65536, size=kk, dtype=np.uint16) for kk in sizes] for _ in range(nl)]
    caches = [fcdp.fcdp_host_cache_alloc(n * S * 2) for _ in range(nl)]
    for H in caches:
        H.numpy(np.uint16)[:] = 0xDEAD
    state = fcdp.CacheState(nl)
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    stg = Arena([n * S * 2, n * S * 2])
    kinds = []
    for it in range(iters):
        for l in range(nl):                                   # ---- forward
            flat = oracle.flatten(params[l], G)
            shards = oracle.split(flat, G)
            dec = {c: state.forward_source(l, c, fcdp.SRC_HOST_DMA) for c in (0, 1)}
            sh = Arena([S * 2] * G)
            out = Arena([kk * 2 for kk in sizes])
            if all(src == fcdp.SRC_DEVICE_SHARDS for src, _ in dec.values()):
                for r in range(G):
                    sh.fill(r, shards[r])                     # everything was gathered
                fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, sh.ptrs(), None, None, out.ptrs(),
                                            fcdp.STORE_NONE, compute, copy)
                fcdp.fcdp_cache_store_node_slice(L, first, n, sh.ptrs(), caches[l], compute, copy)
                kinds.append("miss")
            else:
                assert dec[0] == (fcdp.SRC_HOST_DMA, False) and dec[1] == (fcdp.SRC_DEVICE_SHARDS, True)
                # only the packed trainable values crossed the node boundary: refresh this GPU's
                # slice of H with them, then fetch the slice; the peer's shards hold current values
                d_packed = Arena([L.packed_numel * 2])
                d_packed.fill(0, oracle.pack(flat, sizes, trainable, G))
                for r in range(G):
                    if not first <= r < first + n:
                        sh.fill(r, shards[r])
                fcdp.fcdp_unpack_trainable_node_slice(L, first, n, d_packed.ptr(0), caches[l].dev, copy)
                peers = [None if first <= r < first + n else sh.ptr(r) for r in range(G)]
                fcdp.fcdp_materialize_layer_node_slice(L, first, n, peers, caches[l], stg.ptr(l % 2), out.ptrs(),
                                                       compute, copy)
                kinds.append("refresh")
            torch.cuda.synchronize()
            for t in range(len(sizes)):
                assert np.array_equal(out.get(t, np.uint16), params[l][t]), ("forward", it, l, t)
            assert np.array_equal(caches[l].numpy(np.uint16, n * S), flat[first * S:(first + n) * S]), "host slice is stale"
        for l in range(nl - 1, -1, -1):                       # ---- backward: hits for both classes
            for c in (0, 1):
                assert state.backward_source(l, c, fcdp.SRC_HOST_DMA) == fcdp.SRC_HOST_DMA
            shards = oracle.split(oracle.flatten(params[l], G), G)
            sh = Arena([S * 2] * G)
            for r in range(G):
                if not first <= r < first + n:
                    sh.fill(r, shards[r])
            peers = [None if first <= r < first + n else sh.ptr(r) for r in range(G)]
            out = Arena([kk * 2 for kk in sizes])
            fcdp.fcdp_materialize_layer_node_slice(L, first, n, peers, caches[l], stg.ptr(l % 2), out.ptrs(),
                                                   compute, copy)
            torch.cuda.synchronize()
            for t in range(len(sizes)):
                assert np.array_equal(out.get(t, np.uint16), params[l][t]), ("backward", it, l, t)
        for l in range(nl):                                   # ---- the step changes the trainable tensors only
            for t in range(len(sizes)):
                if trainable[t]:
                    params[l][t] = (params[l][t] + np.uint16(3 + it)).astype(np.uint16)
        state.optimizer_step()
    assert kinds == ["miss"] * nl + ["refresh"] * (nl * (iters - 1))
    for H in caches:
        H.free()
