"""The launch-bound small-layer sweep captured in a HIP graph.

The device-shards materialization, the gradient-shard reduce and the PEFT pack
only launch kernels (no copies, no events, no memsets), so a caller may record
them into a graph and replay it.  The graph is replayed several times with the
inputs rewritten in place by ordinary eager work and a synchronisation between
the replays; every replay is checked against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_06499_amd as fcdp
from paper_2602_06499_amd import synth
from gpu_util import Arena

pytestmark = pytest.mark.gpu


def test_graph_replays_match_the_oracle():
    cfg = synth.CONFIGS["gpt2_small_g4"]
    sizes, G, nl = list(cfg.numel), cfg.G, 3
    tr = [1 if k < 10000 else 0 for k in sizes]          # biases and norms trainable
    L = fcdp.fcdp_layout_build(sizes, tr, G, 2)
    L.prepare()                                         # table upload is not capturable
    S, Np, Pn = L.shard_numel, L.padded_numel, L.packed_numel
    shards = [Arena([S * 2] * G) for _ in range(nl)]
    outs = [Arena([k * 2 for k in sizes]) for _ in range(nl)]
    grads = Arena([S * 4] * G)
    gshard = Arena([S * 4])
    flat = Arena([Np * 2])
    packed = Arena([Pn * 2])
    stream = torch.cuda.Stream()

    def fill(version):
        want = []
        for l in range(nl):
            tensors = synth.layer_params_bf16(cfg, l + 10 * version)
            f = oracle.flatten(tensors, G)
            sh = oracle.split(f, G)
            for r in range(G):
                shards[l].fill(r, sh[r])
            want.append(oracle.materialize_from_shards(sh, sizes))
        parts = [synth.grad_partial_f32(cfg, version, r, S) for r in range(G)]
        for r in range(G):
            grads.fill(r, parts[r])
        flat.fill(0, f)
        return want, oracle.reduce(parts, 0, S, oracle.F32), oracle.pack(f, sizes, tr, G)

    def enqueue():
        for l in range(nl):
            fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, shards[l].ptrs(), None, None,
                                        outs[l].ptrs(), fcdp.STORE_NONE, stream, None)
        fcdp.fcdp_reduce_grad_shard(grads.ptrs(), G, 0, S, fcdp.F32, fcdp.F32, gshard.ptr(0), stream)
        fcdp.fcdp_pack_trainable(L, flat.ptr(0), packed.ptr(0), stream)

    want = fill(0)
    torch.cuda.synchronize()
    enqueue()                                           # eager warm-up of every kernel
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream, capture_error_mode="thread_local"):
        enqueue()
    for version in range(4):
        if version:
            want = fill(version)                        # eager work between replays
        for a in outs + [gshard, packed]:
            a.buf.fill_(0xC3)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for l in range(nl):
            for t in range(len(sizes)):
                assert np.array_equal(outs[l].get(t, np.uint16), want[0][l][t]), (version, l, t)
            outs[l].check_guards()
        assert np.array_equal(gshard.get(0, np.uint32), want[1].view(np.uint32)), version
        assert np.array_equal(packed.get(0, np.uint16), want[2]), version
        gshard.check_guards()
        packed.check_guards()


def test_phased_reduce_in_a_graph():
    """The phased reduce (a persistent grid whose launch shape depends on the
    device's compute-unit count, read once on the host) is an ordinary kernel
    launch: recorded into a graph, replayed four times with the partials
    rewritten in between, every replay the oracle's bits."""
    G, n = 5, 4194304 + 3 * 256 + 2
    grads = Arena([n * 4] * G)
    gshard = Arena([n * 4])
    bshard = Arena([n * 2])
    stream = torch.cuda.Stream()

    def fill(version):
        parts = [synth.grad_partial_f32(synth.CONFIGS["gpt2_small_g4"], 40 + version, r, n) for r in range(G)]
        for r in range(G):
            grads.fill(r, parts[r])
        return oracle.reduce(parts, 0, n, oracle.F32), oracle.reduce(parts, 0, n, oracle.BF16, float(np.float32(0.2)))

    def enqueue():
        fcdp.fcdp_reduce_grad_shard(grads.ptrs(), G, 0, n, fcdp.F32, fcdp.F32, gshard.ptr(0), stream)
        fcdp.fcdp_reduce_grad_shard_scaled(grads.ptrs(), G, 0, n, fcdp.F32, fcdp.BF16, float(np.float32(0.2)),
                                           bshard.ptr(0), stream)

    before = fcdp.fcdp_tuning_get("reduce_phased")
    fcdp.fcdp_tuning_set("reduce_phased", 1)             # both launches take the phased kernel
    try:
        want = fill(0)
        torch.cuda.synchronize()
        enqueue()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream, capture_error_mode="thread_local"):
            enqueue()
    finally:
        fcdp.fcdp_tuning_set("reduce_phased", before)
    for version in range(4):
        if version:
            want = fill(version)
        gshard.buf.fill_(0xC3)
        bshard.buf.fill_(0xC3)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(gshard.get(0, np.uint32), want[0].view(np.uint32)), version
        assert np.array_equal(bshard.get(0, np.uint16), want[1]), version
        gshard.check_guards()
        bshard.check_guards()
