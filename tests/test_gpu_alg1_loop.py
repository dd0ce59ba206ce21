"""Several iterations of Alg. 1's loop on the GPU, with a stand-in optimizer
that rewrites the trainable parameters after every step: whichever source the
dirty flags select (gathered shards on a miss, host cache on a hit, host cache
refreshed by an unpack of the packed trainable values under PEFT), every
forward and backward materialization must equal the current parameters, and
every reduced gradient shard the oracle's."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_06499_amd as fcdp
from paper_2602_06499_amd import synth
from gpu_util import to_dev

pytestmark = pytest.mark.gpu

SIZES = [70001, 640, 640, 130003, 257]


def _bits(t):
    return t.cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("host_mode", [fcdp.SRC_HOST_DMA, fcdp.SRC_HOST_ZEROCOPY, fcdp.SRC_HOST_SCATTER_DMA])
@pytest.mark.parametrize("peft", [False, True])
def test_training_loop_cache_coherence(peft, host_mode):
    nl, G, iters = 3, 4, 4
    trainable = [0, 1, 1, 0, 0] if peft else [1] * len(SIZES)
    L = fcdp.fcdp_layout_build(SIZES, trainable, G, 2)
    L.prepare()
    Np, S = L.padded_numel, L.shard_numel
    g = synth.rng(0, 4242 + peft, synth.KIND_MISC)
    params = [[g.integers(0, 65536, size=k, dtype=np.uint16) for k in SIZES] for _ in range(nl)]
    caches = [fcdp.fcdp_host_cache_alloc(Np * 2) for _ in range(nl)]
    for H in caches:
        H.numpy(np.uint16, Np)[:] = 0xDEAD          # nothing valid is cached yet
    state = fcdp.CacheState(nl)
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    staging = [torch.zeros(Np * 2, dtype=torch.uint8, device="cuda") for _ in range(2)]
    outs = [torch.zeros(k * 2, dtype=torch.uint8, device="cuda") for k in SIZES]
    pk = L.packed_numel
    grad_n = pk // G if peft else S            # this rank's gradient slice
    sources = []

    def check(l, what):
        torch.cuda.synchronize()
        for t, k in enumerate(SIZES):
            assert np.array_equal(_bits(outs[t]), params[l][t]), (what, l, t)
        for o in outs:
            o.zero_()
        torch.cuda.synchronize()

    for it in range(iters):
        # ---- forward
        for l in range(nl):
            flat = oracle.flatten(params[l], G)
            classes = [0, 1] if peft else [1]
            dec = {c: state.forward_source(l, c, host_mode) for c in classes}
            if all(src == fcdp.SRC_DEVICE_SHARDS for src, _ in dec.values()):
                gathered = to_dev(flat)                    # result of the inter-node gather
                ptrs = [gathered.data_ptr() + r * S * 2 for r in range(G)]
                torch.cuda.synchronize()
                fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, ptrs, caches[l], None, outs,
                                            fcdp.STORE_DMA, compute, copy)
                sources.append((it, l, "miss"))
            else:
                if peft:
                    # frozen hits; trainable is dirty: its packed values were gathered,
                    # they refresh H for W_t only, then the whole layer comes from H
                    assert dec[0][0] == host_mode and dec[1][0] == fcdp.SRC_DEVICE_SHARDS
                    packed = to_dev(oracle.pack(flat, SIZES, trainable, G))
                    torch.cuda.synchronize()
                    fcdp.fcdp_unpack_trainable(L, packed, caches[l].dev, copy)
                    sources.append((it, l, "refresh"))
                else:
                    raise AssertionError("full fine-tuning is dirty on every forward")
                fcdp.fcdp_materialize_layer(L, host_mode, None, caches[l], staging[l % 2], outs,
                                            fcdp.STORE_NONE, compute, copy)
            check(l, "forward it%d" % it)
            assert np.array_equal(caches[l].numpy(np.uint16, Np), flat), "host cache is not the current layer"
        # ---- backward
        for l in range(nl - 1, -1, -1):
            for c in ([0, 1] if peft else [1]):
                assert state.backward_source(l, c, host_mode) == host_mode
            fcdp.fcdp_materialize_layer(L, host_mode, None, caches[l], staging[l % 2], outs,
                                        fcdp.STORE_NONE, compute, copy)
            check(l, "backward it%d" % it)
            parts = [synth.grad_partial_f32(synth.CONFIGS["gpt2_small_g4"], it * nl + l, r, grad_n + 5) for r in range(G)]
            d_parts = [to_dev(p) for p in parts]
            d_out = torch.zeros(grad_n * 4, dtype=torch.uint8, device="cuda")
            torch.cuda.synchronize()
            fcdp.fcdp_reduce_grad_shard(d_parts, G, 3, grad_n, fcdp.F32, fcdp.F32, d_out, compute)
            torch.cuda.synchronize()
            assert np.array_equal(d_out.cpu().numpy().view(np.uint32),
                                  oracle.reduce(parts, 3, grad_n, oracle.F32).view(np.uint32))
        # ---- optimizer step: trainable parameters change, their cache goes stale
        for l in range(nl):
            for t, k in enumerate(SIZES):
                if trainable[t]:
                    params[l][t] = g.integers(0, 65536, size=k, dtype=np.uint16)
        state.optimizer_step()
    kinds = [s[2] for s in sources]
    if peft:
        assert kinds[:nl] == ["miss"] * nl and set(kinds[nl:]) == {"refresh"}
    else:
        assert set(kinds) == {"miss"}
    for H in caches:
        H.free()


@pytest.mark.parametrize("tau", [0.0, 0.5, 1.0])
def test_adaptive_gpu_caching(tau):
    """Sec. 4.4: layers whose utilisation at the 'cache on CPU' point is below
    tau stay on the device (no store, no fetch); the others take the host
    cache.  Either way the backward pass sees the layer's parameters, and the
    bytes over the host link are the oracle's."""
    from oracle import alg1
    nl, G = 5, 4
    L = fcdp.fcdp_layout_build(SIZES, None, G, 2)
    L.prepare()
    Np, S = L.padded_numel, L.shard_numel
    g = synth.rng(0, 777, synth.KIND_MISC)
    params = [[g.integers(0, 65536, size=k, dtype=np.uint16) for k in SIZES] for _ in range(nl)]
    caches = [fcdp.fcdp_host_cache_alloc(Np * 2) for _ in range(nl)]
    state = fcdp.CacheState(nl)
    state.set_tau(tau)
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    staging = [torch.zeros(Np * 2, dtype=torch.uint8, device="cuda") for _ in range(2)]
    # one tensor set per layer: a kept layer's tensors must survive until its backward pass
    outs = [[torch.zeros(k * 2, dtype=torch.uint8, device="cuda") for k in SIZES] for _ in range(nl)]

    def util(it, l):
        return 0.2 + 0.15 * l

    want = alg1.replay_adaptive([Np * 2] * nl, util, tau, 2)["iterations"]
    total = 288 << 30
    for it in range(2):
        fcdp.fcdp_link_bytes(True)
        gathered = []
        for l in range(nl):
            src, store = state.forward_source(l, 1, fcdp.SRC_HOST_DMA)
            assert src == fcdp.SRC_DEVICE_SHARDS
            flat = oracle.flatten(params[l], G)
            gathered.append(to_dev(flat))
            ptrs = [gathered[l].data_ptr() + r * S * 2 for r in range(G)]
            torch.cuda.synchronize()
            fcdp.fcdp_materialize_layer(L, src, ptrs, None, None, outs[l], fcdp.STORE_NONE, compute, copy)
            # ... the layer's forward computation would run here ...
            if not state.place(l, int(util(it, l) * total), total):
                fcdp.fcdp_cache_store(L, ptrs, caches[l], fcdp.STORE_DMA, compute, copy)
        torch.cuda.synchronize()
        for l in range(nl - 1, -1, -1):
            src = state.backward_source(l, 1, fcdp.SRC_HOST_DMA)
            if src != fcdp.SRC_DEVICE_RESIDENT:
                for o in outs[l]:
                    o.zero_()           # an offloaded layer was freed after its forward pass
                torch.cuda.synchronize()
            fcdp.fcdp_materialize_layer(L, src, None, caches[l], staging[l % 2], outs[l],
                                        fcdp.STORE_NONE, compute, copy)
            torch.cuda.synchronize()
            for t, k in enumerate(SIZES):
                assert np.array_equal(_bits(outs[l][t]), params[l][t]), (tau, it, l, t)
            assert (src == fcdp.SRC_DEVICE_RESIDENT) == (l in want[it]["kept"])
            state.release(l)
        stored, fetched = fcdp.fcdp_link_bytes()
        assert (stored, fetched) == (want[it]["stored"], want[it]["fetched"])
        for l in range(nl):
            params[l] = [g.integers(0, 65536, size=k, dtype=np.uint16) for k in SIZES]
        state.optimizer_step()
    for H in caches:
        H.free()


@pytest.mark.parametrize("host_mode", [fcdp.SRC_HOST_DMA, fcdp.SRC_HOST_ZEROCOPY])
def test_peft_loop_at_full_layer_size(host_mode):
    """The PEFT loop of Alg. 1 on full-size layers (llama7b_lora_g8: 405 MB of
    bf16 parameters, LoRA r16 on q and v, G = 8), three iterations over two
    layers: a miss with a cache store in the first iteration; from the second
    on the frozen class hits, the trainable class is refreshed by unpacking
    the gathered packed values into the mapped host cache, and the layer is
    materialized from there; every backward pass hits; the trainable gradient
    shard comes from the fused pack + reduce with the mean's scale 1/G.  A
    stand-in optimizer rewrites the LoRA tensors after every step.  Every
    materialization, the cached image and every gradient shard are compared
    with the oracle."""
    cfg = synth.CONFIGS["llama7b_lora_g8"]
    sizes, tr, G = list(cfg.numel), list(cfg.trainable), cfg.G
    nl, iters = 2, 3
    dev = torch.device("cuda:0")
    L = fcdp.fcdp_layout_build(sizes, tr, G, 2)
    L.prepare()
    Np, S, pk = L.padded_numel, L.shard_numel, L.packed_numel
    Sp = pk // G
    params = [synth.layer_params_bf16(cfg, l, lora_b="zero") for l in range(nl)]
    caches = [fcdp.fcdp_host_cache_alloc(Np * 2) for _ in range(nl)]
    for H in caches:
        H.numpy(np.uint16, Np)[:] = 0xDEAD
    state = fcdp.CacheState(nl)
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    staging = [torch.zeros(Np, dtype=torch.int16, device=dev) for _ in range(2)]
    outs = [torch.zeros(max(k, 1), dtype=torch.int16, device=dev) for k in sizes]
    # G flat fp32 gradients of one layer, drawn on the device once; the optimizer
    # stand-in below also rewrites their trainable ranges so every step sums new values
    gen = synth.torch_device_generator(dev, cfg.config_id, 0, synth.KIND_GRAD)
    d_grads = [torch.empty(Np, dtype=torch.float32, device=dev).normal_(0.0, 1e-3, generator=gen) for _ in range(G)]
    h_grads = [d.cpu().numpy() for d in d_grads]
    d_shard = torch.zeros(Sp, dtype=torch.float32, device=dev)
    off = L.offsets
    g = synth.rng(cfg.config_id, 99, synth.KIND_MISC)
    scale = float(np.float32(1.0 / G))
    kinds = []

    def check(l, what):
        torch.cuda.synchronize()
        want = oracle.materialize_from_flat(oracle.flatten(params[l], G), sizes)
        for t, k in enumerate(sizes):
            assert np.array_equal(outs[t][:k].cpu().numpy().view(np.uint16), want[t]), (what, l, t)
        for o in outs:
            o.zero_()
        torch.cuda.synchronize()

    for it in range(iters):
        for l in range(nl):                                       # ---- forward
            flat = oracle.flatten(params[l], G)
            dec = {c: state.forward_source(l, c, host_mode) for c in (0, 1)}
            if all(src == fcdp.SRC_DEVICE_SHARDS for src, _ in dec.values()):
                gathered = to_dev(flat)
                ptrs = [gathered.data_ptr() + r * S * 2 for r in range(G)]
                torch.cuda.synchronize()
                fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, ptrs, caches[l], None, outs,
                                            fcdp.STORE_DMA, compute, copy)
                kinds.append("miss")
            else:
                assert dec[0] == (host_mode, False) and dec[1] == (fcdp.SRC_DEVICE_SHARDS, True)
                packed = to_dev(oracle.pack(flat, sizes, tr, G))     # what the gather of W_t delivers
                torch.cuda.synchronize()
                fcdp.fcdp_unpack_trainable(L, packed, caches[l].dev, copy)
                fcdp.fcdp_materialize_layer(L, host_mode, None, caches[l], staging[l % 2], outs,
                                            fcdp.STORE_NONE, compute, copy)
                kinds.append("refresh")
            check(l, "forward it%d" % it)
            assert np.array_equal(caches[l].numpy(np.uint16, Np), flat), "host cache is not the current layer"
        for l in range(nl - 1, -1, -1):                           # ---- backward
            for c in (0, 1):
                assert state.backward_source(l, c, host_mode) == host_mode
            fcdp.fcdp_materialize_layer(L, host_mode, None, caches[l], staging[l % 2], outs,
                                        fcdp.STORE_NONE, compute, copy)
            check(l, "backward it%d" % it)
            rank = (it * nl + l) % G
            fcdp.fcdp_reduce_trainable_shard_scaled(L, d_grads, rank, fcdp.F32, fcdp.F32, scale, d_shard, compute)
            torch.cuda.synchronize()
            want = oracle.reduce_trainable(h_grads, sizes, tr, G, rank, oracle.F32, scale=scale)
            assert np.array_equal(d_shard.cpu().numpy().view(np.uint32), want.view(np.uint32)), (it, l, rank)
        for l in range(nl):                                       # ---- optimizer step
            for t, k in enumerate(sizes):
                if tr[t]:
                    params[l][t] = g.integers(0, 65536, size=k, dtype=np.uint16)
        for t, k in enumerate(sizes):
            if tr[t]:
                for r in range(G):
                    x = g.standard_normal(k, dtype=np.float32) * np.float32(1e-3)
                    h_grads[r][off[t]:off[t] + k] = x
                    d_grads[r][off[t]:off[t] + k] = torch.from_numpy(x).to(dev)
        state.optimizer_step()
    assert kinds == ["miss"] * nl + ["refresh"] * (nl * (iters - 1))
    for H in caches:
        H.free()
