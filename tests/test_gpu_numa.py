"""Sec. 4.4 "Host Memory Optimization": the cache lives in pinned buffers taken
from the NUMA node local to the GPU.  What one box can show: the numa_node
argument of fcdp_host_cache_alloc takes effect or says why not, and a layer
stored to and fetched from such a buffer has the oracle's bytes."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2602_06499_amd as fcdp
from paper_2602_06499_amd import synth
from gpu_util import Arena

pytestmark = pytest.mark.gpu


def _nodes():
    try:
        return sorted(int(d[4:]) for d in os.listdir("/sys/devices/system/node")
                      if d.startswith("node") and d[4:].isdigit())
    except OSError:
        return []


def test_numa_bound_host_cache_round_trip():
    nodes = _nodes()
    cfg = synth.CONFIGS["gpt2_small_g4"]
    sizes, G = list(cfg.numel), cfg.G
    tensors = synth.layer_params_bf16(cfg, 0)
    flat = oracle.flatten(tensors, G)
    shards = oracle.split(flat, G)
    L = fcdp.fcdp_layout_build(sizes, None, G, 2)
    L.prepare()
    Np = L.padded_numel
    sh = Arena([L.shard_numel * 2] * G)
    for r in range(G):
        sh.fill(r, shards[r])
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    staging = torch.zeros(Np, dtype=torch.int16, device="cuda")
    for node in [-1] + (nodes or [0]):
        H = fcdp.fcdp_host_cache_alloc(Np * 2, numa_node=node)
        note = fcdp.fcdp_last_error()
        # the allocation succeeded; the note is empty (policy applied, or none asked for)
        # or says that the kernel refused the policy
        assert note == "" or "NUMA policy refused" in note or "no NUMA policy call" in note, note
        if node < 0:
            assert note == ""
        assert H.host % 4096 == 0 and H.dev
        H.numpy(np.uint16, Np)[:] = 0xDEAD
        out = Arena([k * 2 for k in sizes])
        torch.cuda.synchronize()
        fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, sh.ptrs(), H, None, out.ptrs(),
                                    fcdp.STORE_DMA, compute, copy)
        torch.cuda.synchronize()
        assert np.array_equal(H.numpy(np.uint16, Np), oracle.cache_store(shards)), node
        want = oracle.materialize_from_flat(flat, sizes)
        for mode in (fcdp.SRC_HOST_DMA, fcdp.SRC_HOST_ZEROCOPY):
            out.buf.fill_(0xC3)
            torch.cuda.synchronize()
            fcdp.fcdp_materialize_layer(L, mode, None, H, staging, out.ptrs(), fcdp.STORE_NONE, compute, copy)
            torch.cuda.synchronize()
            for t in range(len(sizes)):
                assert np.array_equal(out.get(t, np.uint16), want[t]), (node, mode, t)
            out.check_guards()
        if node >= 0 and note == "":
            # where the pages really are: every page of the buffer on the node asked for
            # (numa_maps lists "N<node>=<pages>" per mapping)
            on_node = _pages_on_node(H.host, Np * 2)
            if on_node is not None:
                assert set(on_node) == {node}, on_node
        H.free()
    # a node number beyond the kernel's range is an argument error, not a crash
    with pytest.raises(fcdp.FcdpError) as e:
        fcdp.fcdp_host_cache_alloc(4096, numa_node=1024)
    assert e.value.name == "FCDP_EINVAL"
    # a node this machine does not have: either refused by the kernel (note) or ignored
    missing = (max(nodes) if nodes else 0) + 1
    H = fcdp.fcdp_host_cache_alloc(1 << 20, numa_node=missing)
    assert H.host
    H.free()


def _pages_on_node(addr, nbytes):
    """Nodes that hold pages of the mapping containing addr, from
    /proc/self/numa_maps (None if the file or the mapping is not there)."""
    try:
        with open("/proc/self/numa_maps") as f:
            lines = f.readlines()
    except OSError:
        return None
    best = None
    for line in lines:
        w = line.split()
        try:
            start = int(w[0], 16)
        except (ValueError, IndexError):
            continue
        if start <= addr and (best is None or start > best[0]):
            best = (start, w)
    if best is None:
        return None
    nodes = [int(x[1:].split("=")[0]) for x in best[1] if x.startswith("N") and "=" in x and x[1:].split("=")[0].isdigit()]
    return nodes or None
