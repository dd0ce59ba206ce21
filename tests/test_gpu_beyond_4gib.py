"""Offsets beyond 4 GiB: a layer whose tensors, shards and gradient slices
are each larger than 2^32 bytes, so any 32-bit byte offset in a kernel or in
the host code would wrap.

The layer is too large for the scalar oracle to finish in seconds, so the
byte movers are checked against their definitions evaluated with library
slicing on the device (tensor_t = flat[off_t : off_t + n_t]; H = flat;
packed = the trainable ranges end to end), which the small-size tests tie to
the oracle; the reduction is checked against successive fp32 additions by the
library over the whole slice and against the oracle itself on windows at the
start, across the 4 GiB line and at the ragged end."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_06499_amd as fcdp

pytestmark = pytest.mark.gpu

FOUR_GIB = 1 << 32


def _fill_random(t, seed):
    g = torch.Generator(device=t.device)
    g.manual_seed(seed)
    v = t.view(torch.int32)
    step = 1 << 28
    for i in range(0, v.numel(), step):
        v[i:i + step].random_(-2 ** 31, 2 ** 31 - 1, generator=g)


def _same(a, b, what):
    """torch.equal with a useful message (where the first and last differences are)."""
    assert a.numel() == b.numel(), what
    step, bad, first, last = 1 << 28, 0, -1, -1        # slabs: some library ops stop at 2^31 elements
    for lo in range(0, a.numel(), step):
        x, y = a[lo:lo + step], b[lo:lo + step]
        if not torch.equal(x, y):
            d = (x != y).nonzero().flatten()
            bad += d.numel()
            first = lo + int(d[0]) if first < 0 else first
            last = lo + int(d[-1])
    assert bad == 0, ("%s: %d of %d elements differ, first at %d, last at %d"
                      % (what, bad, a.numel(), first, last))


def test_layer_with_tensors_and_shards_beyond_4gib():
    dev = torch.device("cuda:0")
    sizes = [2 ** 31 + 2 ** 20 + 6, 12345, 2 ** 31 + 5, 3]       # bf16 elements
    G = 2
    L = fcdp.fcdp_layout_build(sizes, [0, 1, 0, 1], G, 2)
    L.prepare()
    N, Np, S = L.numel, L.padded_numel, L.shard_numel
    assert S * 2 > FOUR_GIB and sizes[0] * 2 > FOUR_GIB
    off = L.offsets
    flat = torch.empty(Np + (Np & 1), dtype=torch.int16, device=dev)
    _fill_random(flat, 20260227)
    flat[N:] = 0                                  # the tail padding is zero by construction
    tensors = [torch.zeros(k + (k & 1), dtype=torch.int16, device=dev) for k in sizes]
    H = fcdp.fcdp_host_cache_alloc(Np * 2)
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    shard_ptrs = [flat.data_ptr() + r * S * 2 for r in range(G)]
    torch.cuda.synchronize()
    print("unflatten + store", flush=True)
    fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, shard_ptrs, H, None, tensors,
                                fcdp.STORE_DMA, compute, copy)
    torch.cuda.synchronize()
    for t, k in enumerate(sizes):
        _same(tensors[t][:k], flat[off[t]:off[t] + k], "device shards, tensor %d" % t)
    # the oracle's own index arithmetic at these sizes: its (tensor x shard) segment list
    # says which window of which shard every piece of a tensor comes from; check the first
    # and last 4096 elements of every segment (they straddle the 4 GiB lines) against it
    segs = oracle.segments(sizes, G)
    assert int(segs[:, 4].sum()) == N
    for t_, r_, dst_off, src_off, length in segs.tolist():
        for a in sorted({0, max(0, length - 4096)}):
            n = min(4096, length - a)
            got = tensors[t_][dst_off + a:dst_off + a + n]
            want = flat[r_ * S + src_off + a:r_ * S + src_off + a + n]
            assert torch.equal(got, want), ("oracle segment", t_, r_, a)
    hc = torch.from_numpy(H.numpy(np.int16, Np))
    for lo in range(0, Np, 1 << 29):              # compare in 1 GiB slabs
        hi = min(Np, lo + (1 << 29))
        assert torch.equal(hc[lo:hi], flat[lo:hi].cpu()), ("store", lo)
    # where the 4 GiB lines fall: destination offsets inside tensors 0 and 2,
    # source offsets inside shards 0 and 1 (the latter inside tensor 2)
    e4 = FOUR_GIB // 2                            # element index of byte 2^32
    assert e4 < sizes[0] and e4 < sizes[2] and e4 < S and S < sizes[0]
    assert off[2] < S + e4 < off[2] + sizes[2]
    for mode in (fcdp.SRC_HOST_ZEROCOPY, fcdp.SRC_HOST_DMA, fcdp.SRC_HOST_SCATTER_DMA):
        print("fetch mode", mode, flush=True)
        for t in tensors:
            t.zero_()
        staging = torch.empty(Np, dtype=torch.int16, device=dev) if mode == fcdp.SRC_HOST_DMA else None
        torch.cuda.synchronize()
        fcdp.fcdp_materialize_layer(L, mode, None, H, staging, tensors, fcdp.STORE_NONE, compute, copy)
        torch.cuda.synchronize()
        for t, k in enumerate(sizes):
            _same(tensors[t][:k], flat[off[t]:off[t] + k], "fetch mode %d, tensor %d" % (mode, t))
        del staging
    print("flatten", flush=True)
    back = torch.full((Np,), 0x5A5A, dtype=torch.int16, device=dev)
    torch.cuda.synchronize()                      # the fill runs on torch's stream, the library on `compute`
    fcdp.fcdp_flatten_to_shards(L, tensors, [back.data_ptr() + r * S * 2 for r in range(G)], compute)
    torch.cuda.synchronize()
    _same(back, flat[:Np], "flatten (N = %d, N_pad = %d, S = %d)" % (N, Np, S))
    del back
    print("pack / unpack", flush=True)
    Pn = L.packed_numel
    packed = torch.full((Pn,), 0x5A5A, dtype=torch.int16, device=dev)
    torch.cuda.synchronize()
    fcdp.fcdp_pack_trainable(L, flat, packed, compute)
    torch.cuda.synchronize()
    exp = torch.cat([flat[off[1]:off[1] + sizes[1]], flat[off[3]:off[3] + sizes[3]]])
    _same(packed[:exp.numel()], exp, "pack")
    assert not bool(packed[exp.numel():].any())
    packed.random_(-2 ** 15, 2 ** 15 - 1)
    before = flat.clone()
    torch.cuda.synchronize()
    fcdp.fcdp_unpack_trainable(L, packed, flat, compute)
    torch.cuda.synchronize()
    before[off[1]:off[1] + sizes[1]] = packed[:sizes[1]]
    before[off[3]:off[3] + sizes[3]] = packed[sizes[1]:sizes[1] + sizes[3]]
    _same(flat, before, "unpack")
    H.free()


@pytest.mark.parametrize("e0", [5, 8], ids=["one_tile_per_workgroup", "phased_40_launches"])
def test_gradient_slices_beyond_4gib(e0):
    """e0 = 5 leaves the slices unaligned (the one-tile-per-workgroup kernel);
    e0 = 8 keeps them 16-byte aligned, so the phased kernel runs, as 40
    launches at this size."""
    dev = torch.device("cuda:0")
    G, count = 3, 2 ** 30 + 4099                   # 4 GiB + 16 KiB of fp32 per rank
    parts = [torch.empty(e0 + count + 3, dtype=torch.float32, device=dev) for _ in range(G)]
    for r, p in enumerate(parts):
        _fill_random(p, 77 + r)
        # keep the values finite: clear the top exponent bit
        p.view(torch.int32).bitwise_and_(~(1 << 30))
    out = torch.empty(count, dtype=torch.float32, device=dev)
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    print("reduce fp32 -> fp32", flush=True)
    fcdp.fcdp_reduce_grad_shard(parts, G, e0, count, fcdp.F32, fcdp.F32, out, st)
    torch.cuda.synchronize()
    acc = parts[0][e0:e0 + count].clone()
    for r in range(1, G):
        acc += parts[r][e0:e0 + count]            # one fp32 rounding per add, in rank order
    assert not bool(torch.isnan(acc).any())     # inputs were kept below 2.0
    _same(out.view(torch.int32), acc.view(torch.int32), "fp32 shard against successive library adds")
    # the oracle on windows at the start, across the 4 GiB line, and at the ragged end
    for centre in (3000, (FOUR_GIB // 4) - e0, count - 3000):
        lo, hi = centre - 3000, min(count, centre + 3000)
        wp = [p[e0 + lo:e0 + hi].cpu().numpy() for p in parts]
        want = oracle.reduce(wp, 0, hi - lo, oracle.F32)
        got = out[lo:hi].cpu().numpy()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), centre
    print("reduce fp32 -> bf16", flush=True)
    outb = torch.empty(count + (count & 1), dtype=torch.int16, device=dev)
    fcdp.fcdp_reduce_grad_shard(parts, G, e0, count, fcdp.F32, fcdp.BF16, outb, st)
    torch.cuda.synchronize()
    lo, hi = count - 6000, count
    wp = [p[e0 + lo:e0 + hi].cpu().numpy() for p in parts]
    want = oracle.reduce(wp, 0, hi - lo, oracle.BF16)
    got = outb[lo:hi].cpu().numpy().view(np.uint16)
    assert np.array_equal(got, want)
    wantb = acc.to(torch.bfloat16).view(torch.int16)     # RNE cast by the library
    _same(outb[:count], wantb, "bf16 shard against the library cast")
