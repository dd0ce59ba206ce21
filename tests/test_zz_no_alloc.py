"""The allocation-free staged fetch, fcdp_materialize_layer_static, through the
C ABI: its tensors against those of the existing staged fetch
(fcdp_materialize_layer with FCDP_SRC_HOST_DMA and a caller staging buffer),
bit for bit, and both against the oracle.  Two calls in a row share the
library's static staging array, the second with a smaller layer, so bytes the
first call left in the array lie right behind what the second call reads."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_06499_amd as fcdp
from paper_2602_06499_amd import synth
from gpu_util import Arena

pytestmark = pytest.mark.gpu


def _layer(cfg_sizes, G, seed):
    g = synth.rng(0, seed, synth.KIND_MISC, 77)
    tensors = [g.integers(0, 65536, size=k, dtype=np.uint16) for k in cfg_sizes]
    flat = oracle.flatten(tensors, G)
    return tensors, flat


def _fetch_both_ways(sizes, G, seed, compute, copy):
    """Returns nothing; asserts static == staged == oracle for one layer."""
    tensors, flat = _layer(sizes, G, seed)
    want = oracle.materialize_from_flat(flat, sizes)
    L = fcdp.fcdp_layout_build(sizes, None, G, 2)
    L.prepare()
    Np = L.padded_numel
    assert Np * 2 <= fcdp.STATIC_STAGING_BYTES
    H = fcdp.fcdp_host_cache_alloc(max(Np * 2, 16))
    H.numpy(np.uint16, Np)[:] = flat
    staging = torch.full((max(Np, 8),), 0x5A5A, dtype=torch.int16, device="cuda")
    ref = Arena([k * 2 for k in sizes])
    got = Arena([k * 2 for k in sizes])
    torch.cuda.synchronize()
    fcdp.fcdp_materialize_layer(L, fcdp.SRC_HOST_DMA, None, H, staging, ref.ptrs(),
                                fcdp.STORE_NONE, compute, copy)
    fcdp.fcdp_materialize_layer_static(L, H, got.ptrs(), compute, copy)
    torch.cuda.synchronize()
    for t, k in enumerate(sizes):
        a, b = got.get(t, np.uint16), ref.get(t, np.uint16)
        assert np.array_equal(a, b), ("static vs staged", t)
        assert np.array_equal(a, want[t]), ("static vs oracle", t)
    got.check_guards()
    ref.check_guards()
    H.free()


def test_static_fetch_matches_staged_fetch_twice_second_smaller():
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    cfg = synth.CONFIGS["gpt2_small_g4"]
    # first: the GPT-2-small layer (14.2 MB of the 32 MiB array), several tiles and odd tensors
    _fetch_both_ways(list(cfg.numel), cfg.G, 1, compute, copy)
    # second, right after it and smaller: ragged sizes, a straddled shard boundary, an empty tensor
    _fetch_both_ways([300001, 7, 0, 65537, 131075, 1], 3, 2, compute, copy)
    # third: back to back on ONE stream pair without a host sync in between, the
    # second call's copy must wait for the first call's scatter
    sizes_a, sizes_b = [50000, 33, 70001], [4099, 12345]
    ta, fa = _layer(sizes_a, 4, 3)
    tb, fb = _layer(sizes_b, 2, 4)
    La = fcdp.fcdp_layout_build(sizes_a, None, 4, 2)
    Lb = fcdp.fcdp_layout_build(sizes_b, None, 2, 2)
    La.prepare()
    Lb.prepare()
    Ha = fcdp.fcdp_host_cache_alloc(La.padded_numel * 2)
    Hb = fcdp.fcdp_host_cache_alloc(Lb.padded_numel * 2)
    Ha.numpy(np.uint16, La.padded_numel)[:] = fa
    Hb.numpy(np.uint16, Lb.padded_numel)[:] = fb
    oa, ob = Arena([k * 2 for k in sizes_a]), Arena([k * 2 for k in sizes_b])
    torch.cuda.synchronize()
    fcdp.fcdp_materialize_layer_static(La, Ha, oa.ptrs(), compute, copy)
    fcdp.fcdp_materialize_layer_static(Lb, Hb, ob.ptrs(), copy, compute)   # streams swapped on purpose
    torch.cuda.synchronize()
    for t in range(len(sizes_a)):
        assert np.array_equal(oa.get(t, np.uint16), ta[t])
    for t in range(len(sizes_b)):
        assert np.array_equal(ob.get(t, np.uint16), tb[t])
    oa.check_guards()
    ob.check_guards()
    Ha.free()
    Hb.free()


def test_static_fetch_rejects_what_it_cannot_do():
    # a layer one quantum beyond the array: FCDP_ESIZE, nothing enqueued
    big = fcdp.STATIC_STAGING_BYTES // 2 + 64
    L = fcdp.fcdp_layout_build([big], None, 1, 2)
    L.prepare()
    out = torch.zeros(big, dtype=torch.int16, device="cuda")
    H = fcdp.fcdp_host_cache_alloc(L.padded_numel * 2)
    with pytest.raises(fcdp.FcdpError) as e:
        fcdp.fcdp_materialize_layer_static(L, H, [out], None, None)
    assert e.value.name == "FCDP_ESIZE" and "FCDP_STATIC_STAGING_BYTES" in str(e.value)
    # exactly the array's size is accepted
    fit = fcdp.STATIC_STAGING_BYTES // 2
    Lf = fcdp.fcdp_layout_build([fit], None, 1, 2)
    Lf.prepare()
    Hf = fcdp.fcdp_host_cache_alloc(fit * 2)
    Hf.numpy(np.uint16, fit)[:] = np.arange(fit, dtype=np.uint64).astype(np.uint16)
    outf = torch.zeros(fit, dtype=torch.int16, device="cuda")
    torch.cuda.synchronize()
    fcdp.fcdp_materialize_layer_static(Lf, Hf, [outf], None, None)
    torch.cuda.synchronize()
    assert np.array_equal(outf.cpu().numpy().view(np.uint16), Hf.numpy(np.uint16, fit))
    # a layout that was never prepared: FCDP_ESTATE (the call uploads nothing)
    Lu = fcdp.fcdp_layout_build([4096], None, 1, 2)
    Hu = fcdp.fcdp_host_cache_alloc(4096 * 2)
    o = torch.zeros(4096, dtype=torch.int16, device="cuda")
    with pytest.raises(fcdp.FcdpError) as e:
        fcdp.fcdp_materialize_layer_static(Lu, Hu, [o], None, None)
    assert e.value.name == "FCDP_ESTATE"
    with pytest.raises(fcdp.FcdpError) as e:
        fcdp.fcdp_materialize_layer_static(Lf, None, [outf], None, None)
    assert e.value.name == "FCDP_EINVAL"
    for h in (H, Hf, Hu):
        h.free()
