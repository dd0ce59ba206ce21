"""The debug poison: with the knob on, outputs are filled with a NaN pattern
before the work that writes them is enqueued.  Results must not change, and
the fill must really happen where the header says."""
import time

import numpy as np
import pytest
import torch

import oracle
import paper_2602_06499_amd as fcdp
from paper_2602_06499_amd import synth
from gpu_util import Arena

import test_gpu_alg1_loop as loop
import test_gpu_stream_order as order
import test_gpu_node_slice as node

pytestmark = pytest.mark.gpu


@pytest.fixture
def poison():
    fcdp.fcdp_tuning_set("debug_poison", 1)
    try:
        yield
    finally:
        fcdp.fcdp_tuning_set("debug_poison", 0)


@pytest.mark.parametrize("host_mode", [fcdp.SRC_HOST_DMA, fcdp.SRC_HOST_ZEROCOPY, fcdp.SRC_HOST_SCATTER_DMA])
def test_training_loop_under_poison(poison, host_mode):
    loop.test_training_loop_cache_coherence(True, host_mode)
    loop.test_training_loop_cache_coherence(False, host_mode)


def test_adaptive_caching_under_poison(poison):
    loop.test_adaptive_gpu_caching(0.5)


def test_stream_order_under_poison(poison):
    order.test_scatter_waits_for_a_late_fetch()
    order.test_host_sources_wait_for_a_late_store(fcdp.SRC_HOST_ZEROCOPY)
    order.test_store_waits_for_a_late_producer(fcdp.STORE_DMA)
    order.test_staging_reuse_waits_for_a_late_scatter()
    order.test_scatter_dma_waits_for_earlier_readers()


def test_node_slice_under_poison(poison):
    """The slice store and fetch with the fills and the extent checks on: same
    bytes, and the arenas' guards (checked inside) stay untouched."""
    node.test_node_slice_store_and_fetch(8, 2, 4, 5, 50000)
    node.test_node_slice_store_and_fetch(16, 4, 2, 20, 90000)
    node.test_node_slice_backward_sweep_two_staging_slices()
    node.test_node_slice_training_loop_stays_coherent()


def test_poison_is_written_first(poison):
    """The fill is real: with `copy` held back, the scatter of a DMA fetch
    cannot start, so a snapshot of the tensors taken meanwhile must show the
    pattern everywhere; afterwards the tensors hold the layer."""
    sizes, G = [70000, 5, 65536, 9], 4
    L = fcdp.fcdp_layout_build(sizes, None, G, 2)
    L.prepare()       # else the call below uploads the tables, a synchronous copy that may queue behind the held-back stream
    Np = L.padded_numel
    tensors = [synth.rng(0, 3, synth.KIND_MISC, t).integers(0, 65536, size=k, dtype=np.uint16)
               for t, k in enumerate(sizes)]
    flat = oracle.flatten(tensors, G)
    H = fcdp.fcdp_host_cache_alloc(Np * 2)
    H.numpy(np.uint16, Np)[:] = flat
    out = Arena([k * 2 for k in sizes])
    staging = Arena([Np * 2])
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    # Streams share a few hardware queues, so a snapshot stream may sit behind the
    # held-back `copy` or behind `compute`'s wait for it, depending on how many streams
    # the process made before; eight side streams cover every queue, and the snapshots
    # that do run meanwhile must show the pattern
    sides = [torch.cuda.Stream() for _ in range(8)]
    snaps = [torch.empty_like(out.buf) for _ in sides]
    torch.cuda.synchronize()
    with torch.cuda.stream(copy):
        torch.cuda._sleep(order.SPIN)
    fcdp.fcdp_materialize_layer(L, fcdp.SRC_HOST_DMA, None, H, staging.ptr(0), out.ptrs(),
                                fcdp.STORE_NONE, compute, copy)
    time.sleep(0.003)             # the fill runs at once on the idle stream (microseconds)
    for side, snap in zip(sides, snaps):
        with torch.cuda.stream(side):
            snap.copy_(out.buf)   # the scatter is still blocked behind `copy`
    torch.cuda.synchronize()
    poisoned = 0
    for snap in snaps:
        h = snap.cpu().numpy()
        states = []
        for (o, nb), want in zip(out.ranges, tensors):
            got = h[o:o + nb].view(np.uint16)
            if np.all(got == 0x7FC1):
                states.append("poison")
            else:
                # a snapshot that ran late sees the layer, or, if it ran beside the scatter,
                # the layer where the scatter has been and the pattern elsewhere; never stale bytes
                assert np.all((got == want) | (got == 0x7FC1)), "tensor holds neither the pattern nor the layer"
                states.append("layer")
        poisoned += all(st == "poison" for st in states)
    assert poisoned >= 1, "no snapshot saw the tensors poisoned ahead of the fetch"
    for t, k in enumerate(sizes):
        assert np.array_equal(out.get(t, np.uint16), tensors[t])
    out.check_guards()
    staging.check_guards()
    H.free()


def test_debug_mode_refuses_buffers_that_are_too_small(poison):
    """No sizes cross the C boundary; with debug_poison on the library looks
    each device buffer up in the runtime's allocation table and refuses one
    that ends before the documented size (FCDP_ESIZE, nothing enqueued).
    Buffers here come straight from hipMalloc, one allocation each, so the
    short one really is short."""
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipMalloc.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_size_t]
    hip.hipFree.argtypes = [ctypes.c_void_p]

    def dmalloc(nbytes):
        p = ctypes.c_void_p()
        assert hip.hipMalloc(ctypes.byref(p), nbytes) == 0
        return p.value

    sizes, G = [4096, 1000], 2
    L = fcdp.fcdp_layout_build(sizes, None, G, 2)
    L.prepare()
    S = L.shard_numel
    shards = [dmalloc(S * 2) for _ in range(G)]
    good = [dmalloc(k * 2) for k in sizes]
    short = [good[0], dmalloc(sizes[1] * 2 - 512)]       # 256 elements short
    torch.cuda.synchronize()
    with pytest.raises(fcdp.FcdpError) as e:
        fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, shards, None, None, short)
    assert e.value.name == "FCDP_ESIZE" and "a tensor" in str(e.value)
    with pytest.raises(fcdp.FcdpError) as e:
        fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, [shards[0], short[1]], None, None, good)
    assert e.value.name == "FCDP_ESIZE" and "a shard" in str(e.value)
    fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, shards, None, None, good)   # right sizes pass
    parts = [dmalloc(4000 * 4), dmalloc(4000 * 4 - 256)]
    out = dmalloc(4000 * 4)
    with pytest.raises(fcdp.FcdpError) as e:
        fcdp.fcdp_reduce_grad_shard(parts, 2, 0, 4000, fcdp.F32, fcdp.F32, out)
    assert e.value.name == "FCDP_ESIZE" and "a partial" in str(e.value)
    fcdp.fcdp_reduce_grad_shard(parts, 2, 0, 3900, fcdp.F32, fcdp.F32, out)              # fits: passes
    torch.cuda.synchronize()
    for p in shards + good + [short[1], out] + parts:
        hip.hipFree(p)
