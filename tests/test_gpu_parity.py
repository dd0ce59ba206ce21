"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Bit-exact for every copy/pack/index operation and
for the rank-order fp32 reduction (NaN lanes: NaN-ness only)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_06499_amd as fcdp
from paper_2602_06499_amd import synth
from gpu_util import Arena, to_dev, to_host

pytestmark = pytest.mark.gpu


def _rand_tensors(seed, sizes, dtype):
    g = synth.rng(0, seed, synth.KIND_MISC, 21)
    info = np.iinfo(dtype)
    return [g.integers(0, int(info.max) + 1, size=k, dtype=dtype) for k in sizes]


def _layer_cases():
    cases = []
    for G in (1, 2, 3, 4, 8, 16, 32, 64):
        for k, esz in enumerate((2, 4)):
            sizes = synth.random_layer(4000 + G * 3 + k, T=7 + G % 5, max_numel=70000)
            cases.append(("rand_G%d_e%d" % (G, esz), sizes, G, esz))
    cases.append(("tiny_padding_only_shards", [3, 0, 1], 8, 2))
    cases.append(("single_element", [1], 4, 2))
    cases.append(("zeros_and_one", [0, 0, 5, 0], 3, 4))
    cases.append(("aligned_multi_tile", [8 * 40000, 8 * 1000, 8 * 123457], 4, 2))
    cases.append(("odd_multi_tile", [300001, 7, 65537, 131075], 3, 2))
    cases.append(("many_tensors", [(i * 37) % 501 for i in range(600)], 5, 2))
    return cases


CASES = _layer_cases()


@pytest.mark.parametrize("name,sizes,G,esz", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("contiguous", [False, True])
def test_unflatten_and_flatten(name, sizes, G, esz, contiguous):
    dt = np.uint16 if esz == 2 else np.uint32
    tensors = _rand_tensors(len(sizes) + G, sizes, dt)
    flat = oracle.flatten(tensors, G)
    shards = oracle.split(flat, G)
    want = oracle.materialize_from_shards(shards, sizes)
    L = fcdp.fcdp_layout_build(sizes, None, G, esz)
    S = L.shard_numel
    assert S == shards[0].size
    if contiguous:
        sh_arena = Arena([S * esz * G])
        sh_arena.fill(0, flat)
        sh_ptrs = [sh_arena.ptr(0) + r * S * esz for r in range(G)]
    else:
        sh_arena = Arena([S * esz] * G)
        for r in range(G):
            sh_arena.fill(r, shards[r])
        sh_ptrs = sh_arena.ptrs()
    out = Arena([k * esz for k in sizes])
    fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, sh_ptrs, None, None,
                                out.ptrs(), False, None, None)
    torch.cuda.synchronize()
    for t in range(len(sizes)):
        assert np.array_equal(out.get(t, dt), want[t]), (name, t)
    out.check_guards()
    sh_arena.check_guards()
    # inverse: tensors -> shards with zero tail padding
    back = Arena([S * esz] * G)
    fcdp.fcdp_flatten_to_shards(L, out.ptrs(), back.ptrs(), None)
    torch.cuda.synchronize()
    for r in range(G):
        assert np.array_equal(back.get(r, dt), shards[r]), (name, r)
    back.check_guards()


@pytest.mark.parametrize("name,sizes,G,esz", CASES[::3] + CASES[-6:], ids=[c[0] for c in CASES[::3] + CASES[-6:]])
def test_host_cache_store_and_fetch(name, sizes, G, esz):
    """Store on a miss, then both host sources give the same tensors as the
    device source (the cache-hit path equals the cache-miss path)."""
    dt = np.uint16 if esz == 2 else np.uint32
    tensors = _rand_tensors(len(sizes) * 3 + G, sizes, dt)
    flat = oracle.flatten(tensors, G)
    shards = oracle.split(flat, G)
    want = oracle.materialize_from_shards(shards, sizes)
    L = fcdp.fcdp_layout_build(sizes, None, G, esz)
    S, Np = L.shard_numel, L.padded_numel
    sh = Arena([S * esz] * G)
    for r in range(G):
        sh.fill(r, shards[r])
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    H = fcdp.fcdp_host_cache_alloc(max(Np * esz, 16))
    H.numpy(np.uint8)[:] = 0x77
    out0 = Arena([k * esz for k in sizes])
    torch.cuda.synchronize()    # arenas were filled on torch's stream
    fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, sh.ptrs(), H, None,
                                out0.ptrs(), True, compute, copy)
    torch.cuda.synchronize()
    assert np.array_equal(H.numpy(dt, Np), oracle.cache_store(shards))
    assert np.array_equal(H.numpy(dt, Np), flat)
    for mode in (fcdp.SRC_HOST_DMA, fcdp.SRC_HOST_ZEROCOPY, fcdp.SRC_HOST_SCATTER_DMA):
        out = Arena([k * esz for k in sizes])
        staging = Arena([Np * esz]) if mode == fcdp.SRC_HOST_DMA else None
        torch.cuda.synchronize()
        fcdp.fcdp_materialize_layer(L, mode, None, H,
                                    staging.ptr(0) if staging else None,
                                    out.ptrs(), False, compute, copy)
        torch.cuda.synchronize()
        for t in range(len(sizes)):
            assert np.array_equal(out.get(t, dt), want[t]), (name, mode, t)
        out.check_guards()
        if staging:
            staging.check_guards()
    H.free()


REDUCE_CASES = [
    # G, count, elem_offset, in, out
    (1, 1000, 0, oracle.F32, oracle.F32),
    (2, 4099, 0, oracle.F32, oracle.F32),
    (3, 70001, 5, oracle.F32, oracle.BF16),
    (4, 1 << 18, 0, oracle.F32, oracle.F32),
    (7, 33333, 3, oracle.F32, oracle.F32),
    (8, 300007, 0, oracle.F32, oracle.BF16),
    (9, 12345, 1, oracle.F32, oracle.F32),
    (15, 5000, 2, oracle.F32, oracle.BF16),
    (16, 65536 + 3, 0, oracle.F32, oracle.F32),
    (17, 40000, 7, oracle.F32, oracle.F32),
    (32, 100003, 0, oracle.F32, oracle.BF16),
    (33, 2049, 0, oracle.F32, oracle.F32),
    (64, 30001, 11, oracle.F32, oracle.F32),
    (1, 777, 1, oracle.BF16, oracle.BF16),
    (4, 50001, 0, oracle.BF16, oracle.F32),
    (8, 262147, 3, oracle.BF16, oracle.BF16),
    (32, 9999, 5, oracle.BF16, oracle.F32),
    (5, 3, 0, oracle.F32, oracle.F32),
    (5, 0, 0, oracle.F32, oracle.F32),
]


def _cmp_reduce(got, want, out_dtype):
    if out_dtype == oracle.F32:
        nan = np.isnan(want)
        assert np.array_equal(np.isnan(got), nan)
        assert np.array_equal(got.view(np.uint32)[~nan], want.view(np.uint32)[~nan])
    else:
        nan = ((want & 0x7F80) == 0x7F80) & ((want & 0x7F) != 0)
        gnan = ((got & 0x7F80) == 0x7F80) & ((got & 0x7F) != 0)
        assert np.array_equal(gnan, nan)
        assert np.array_equal(got[~nan], want[~nan])


@pytest.mark.parametrize("G,count,e0,in_dt,out_dt", REDUCE_CASES)
def test_reduce_parity(G, count, e0, in_dt, out_dt):
    g = synth.rng(0, 900 + G, synth.KIND_GRAD, count % 1000)
    total = e0 + count + 13
    parts = []
    for r in range(G):
        x = g.standard_normal(total, dtype=np.float32) * np.float32(10.0 ** int(g.integers(-5, 2)))
        parts.append(x if in_dt == oracle.F32 else synth.to_bf16_bits(x))
    want = oracle.reduce(parts, e0, count, out_dt)
    ies = 4 if in_dt == oracle.F32 else 2
    oes = 4 if out_dt == oracle.F32 else 2
    arena = Arena([total * ies] * G)
    for r in range(G):
        arena.fill(r, parts[r])
    out = Arena([count * oes])
    fcdp.fcdp_reduce_grad_shard(arena.ptrs(), G, e0, count, in_dt, out_dt, out.ptr(0), None)
    torch.cuda.synchronize()
    got = out.get(0, np.float32 if out_dt == oracle.F32 else np.uint16)
    _cmp_reduce(got, want, out_dt)
    out.check_guards()


def test_reduce_special_values_and_order():
    """Inf, NaN, signed zeros, denormals, cancellation: same bits as the oracle."""
    G = 6
    specials = np.array([0x00000000, 0x80000000, 0x00000001, 0x80000001, 0x007FFFFF,
                         0x00800000, 0x7F7FFFFF, 0xFF7FFFFF, 0x7F800000, 0xFF800000,
                         0x7FC00000, 0x3F800000, 0xBF800000, 0x4B800000, 0x4B800001,
                         0x33800000, 0x4CBEBC20, 0xCCBEBC20], dtype=np.uint32)
    g = synth.rng(0, 77, synth.KIND_MISC)
    n = 50000
    parts = [specials[g.integers(0, specials.size, size=n)].view(np.float32).copy() for _ in range(G)]
    # order-sensitive columns: (2^24 + 1) + 1 and (1e8 + 1) - 1e8
    parts[0][:2] = [2.0 ** 24, 1e8]
    parts[1][:2] = [1.0, 1.0]
    parts[2][:2] = [1.0, -1e8]
    for r in range(3, G):
        parts[r][:2] = 0.0
    # a column of -0.0 must stay -0.0
    for r in range(G):
        parts[r][2] = -0.0
    for out_dt in (oracle.F32, oracle.BF16):
        with np.errstate(all="ignore"):
            want = oracle.reduce(parts, 0, n, out_dt)
        arena = Arena([n * 4] * G)
        for r in range(G):
            arena.fill(r, parts[r])
        out = Arena([n * (4 if out_dt == oracle.F32 else 2)])
        fcdp.fcdp_reduce_grad_shard(arena.ptrs(), G, 0, n, fcdp.F32, out_dt, out.ptr(0), None)
        torch.cuda.synchronize()
        got = out.get(0, np.float32 if out_dt == oracle.F32 else np.uint16)
        _cmp_reduce(got, want, out_dt)
        if out_dt == oracle.F32:
            assert got[0] == np.float32(2.0 ** 24) and got[1] == 0.0
            assert got.view(np.uint32)[2] == 0x80000000


def test_bf16_rounding_all_upper_halves():
    """G = 1 reduce with bf16 output is the rounding alone: every upper half
    with 288 lower halves around the rounding edges."""
    lows = np.concatenate([np.arange(0, 64), np.arange(0x7FE0, 0x8020), np.arange(0xFFC0, 0x10000),
                           np.arange(0x4000, 0x4040), np.arange(0xBFE0, 0xC000)]).astype(np.uint32)
    assert lows.size == 288
    hi = (np.arange(65536, dtype=np.uint32) << 16)
    u = (hi[:, None] | lows[None, :]).reshape(-1)
    x = u.view(np.float32)
    want = oracle.bf16_rne(x)
    d = to_dev(x)
    out = torch.empty(x.size * 2, dtype=torch.uint8, device="cuda")
    fcdp.fcdp_reduce_grad_shard([d], 1, 0, x.size, fcdp.F32, fcdp.BF16, out, None)
    torch.cuda.synchronize()
    got = to_host(out, np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], want[~nan])
    # NaN stays NaN with its sign
    assert np.all((got[nan] & 0x7F80) == 0x7F80) and np.all((got[nan] & 0x7F) != 0)
    assert np.array_equal(got[nan] >> 15, want[nan] >> 15)


def test_bf16_rounding_all_lower_halves():
    """The other direction of the test above: every one of the 65,536 lower
    halves under 2,048 upper halves (both signs, all 256 exponents, the
    mantissa patterns 0x00, 0x01, 0x7E, 0x7F: even and odd last kept bit, and
    the carries into the exponent and into infinity).  The rounding decision
    depends on the lower half and the last kept bit only, the carry on the
    rest, so the two tests together cover every case of the 2^32 inputs."""
    uppers = np.array([(s << 15) | (e << 7) | m for s in (0, 1) for e in range(256)
                       for m in (0x00, 0x01, 0x7E, 0x7F)], dtype=np.uint32)
    lows = np.arange(65536, dtype=np.uint32)
    step = 256                                     # upper halves per chunk: 16.8 M inputs
    d_out = torch.empty(step * 65536, dtype=torch.int16, device="cuda")
    for c in range(0, uppers.size, step):
        u = ((uppers[c:c + step, None] << 16) | lows[None, :]).reshape(-1)
        x = u.view(np.float32)
        want = oracle.bf16_rne(x)
        d = to_dev(x)
        torch.cuda.synchronize()
        fcdp.fcdp_reduce_grad_shard([d], 1, 0, x.size, fcdp.F32, fcdp.BF16, d_out, None)
        torch.cuda.synchronize()
        got = d_out.cpu().numpy().view(np.uint16)
        nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
        assert np.array_equal(got[~nan], want[~nan]), c
        if nan.any():
            g = got[nan]
            assert np.all((g & 0x7F80) == 0x7F80) and np.all((g & 0x7F) != 0), c
            assert np.array_equal(g >> 15, want[nan] >> 15), c


def test_reduce_in_place_and_all_ranks():
    """Every rank's shard in turn; the G shards concatenate to the full sum.
    Rank r reduces in place into its own partial's slice."""
    cfg = synth.CONFIGS["gpt2_small_g4"]
    G, S = 4, 20480 + 64
    parts = [synth.grad_partial_f32(cfg, 0, r, G * S) for r in range(G)]
    want = np.concatenate([oracle.reduce(parts, r * S, S, oracle.F32) for r in range(G)])
    arena = Arena([G * S * 4] * G)
    for r in range(G):
        arena.fill(r, parts[r])
    for r in range(G):
        fcdp.fcdp_reduce_grad_shard(arena.ptrs(), G, r * S, S, fcdp.F32, fcdp.F32,
                                    arena.ptr(r) + r * S * 4, None)
    torch.cuda.synchronize()
    got = np.concatenate([arena.get(r, np.float32)[r * S:(r + 1) * S] for r in range(G)])
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    arena.check_guards()


# The phased reduce (persistent waves that keep their sums in registers and
# store them after their last load) only runs on aligned slices of at least 8
# steps per wave (2.1 M fp32 / 4.2 M bf16 elements on 256 compute units), so
# the small cases above never reach it.  Counts here sit just above that
# threshold, with ragged tails (count % 4, a partial last step), every
# remainder of G modulo the load group, and, for G = 2, more than one launch
# (beyond 27.3 M elements).  Knob 1 forces the phased kernel from 8 steps per
# wave on; knob 2 (the default) leaves the choice to the rule, which wants
# long launches.
PHASED_CASES = [
    # G, count, elem_offset, in, out, knob
    (1, 2097152, 0, oracle.F32, oracle.F32, 1),          # exactly 8 steps per wave
    (1, 2097152 - 256, 0, oracle.F32, oracle.F32, 1),    # one step short: the other kernel
    (6, 4194304, 0, oracle.F32, oracle.F32, 1),
    (2, 4194304 + 255, 0, oracle.F32, oracle.BF16, 1),   # partial last step, count % 4 = 3
    (3, 4300001, 4, oracle.F32, oracle.F32, 1),
    (3, 13000001, 4, oracle.F32, oracle.F32, 2),         # the rule takes it (fp32 in and out, G >= 3, 0.48 of a full launch)
    (5, 4200002, 8, oracle.F32, oracle.F32, 1),
    (8, 4194304 + 64 * 4 * 7 + 2, 0, oracle.F32, oracle.F32, 1),
    (8, 20000003, 0, oracle.F32, oracle.BF16, 2),        # the rule: one wave per SIMD
    (16, 14000005, 8, oracle.BF16, oracle.BF16, 2),      # the rule: half a launch, so two waves per SIMD
    (9, 4250000, 12, oracle.F32, oracle.BF16, 1),
    (12, 4200003, 0, oracle.F32, oracle.BF16, 1),
    (15, 4194304 + 1, 0, oracle.F32, oracle.F32, 1),
    (23, 4210000, 16, oracle.BF16, oracle.F32, 1),       # bf16 in, just above its 4.2 M threshold
    (4, 4100000, 8, oracle.BF16, oracle.BF16, 1),        # bf16 in, below it: the other kernel
    (16, 8388608 + 517, 8, oracle.BF16, oracle.BF16, 1), # bf16 in, 8 elements per lane and step
    (13, 8400007, 0, oracle.BF16, oracle.F32, 1),
    (7, 8388608 + 9, 16, oracle.BF16, oracle.BF16, 1),
    (32, 4300000, 0, oracle.F32, oracle.BF16, 1),
    (64, 4194304 + 260, 0, oracle.F32, oracle.F32, 1),
    (2, 27262976 + 300001, 0, oracle.F32, oracle.F32, 1),   # two launches
    (2, 3 * 27262976 + 77, 0, oracle.BF16, oracle.BF16, 1), # bf16 in, four launches
    (8, 22544384 - 1001, 0, oracle.F32, oracle.F32, 2),     # 86 steps per wave: the rotated start
    (8, 27262976 + 1500001, 0, oracle.F32, oracle.BF16, 2), # a full launch, the rest by one tile per workgroup
    (8, 2 * 27262976 + 21000003, 4, oracle.F32, oracle.F32, 2), # two full launches and a third of 0.77 of one
    (4, 4300000, 3, oracle.F32, oracle.F32, 1),          # slices not 16-byte aligned: the other kernel
]


@pytest.mark.parametrize("G,count,e0,in_dt,out_dt,knob", PHASED_CASES)
def test_reduce_phased_parity(G, count, e0, in_dt, out_dt, knob):
    g = synth.rng(0, 1900 + G, synth.KIND_GRAD, count % 1000)
    total = e0 + count + 5
    parts = []
    for r in range(G):
        x = g.standard_normal(total, dtype=np.float32) * np.float32(10.0 ** int(g.integers(-5, 2)))
        parts.append(x if in_dt == oracle.F32 else synth.to_bf16_bits(x))
    ies = 4 if in_dt == oracle.F32 else 2
    oes = 4 if out_dt == oracle.F32 else 2
    arena = Arena([total * ies] * G)
    for r in range(G):
        arena.fill(r, parts[r])
    out = Arena([count * oes])
    before = fcdp.fcdp_tuning_get("reduce_phased")
    try:
        fcdp.fcdp_tuning_set("reduce_phased", knob)
        # the knob value 1 takes the shape the rule gives (one wave per SIMD for full
        # load groups); G = 16 and 64 also run the two-wave shape below
        for scale in (None, float(np.float32(1.0 / G))):
            want = oracle.reduce(parts, e0, count, out_dt, scale)
            if scale is None:
                fcdp.fcdp_reduce_grad_shard(arena.ptrs(), G, e0, count, in_dt, out_dt, out.ptr(0), None)
            else:
                fcdp.fcdp_reduce_grad_shard_scaled(arena.ptrs(), G, e0, count, in_dt, out_dt, scale,
                                                   out.ptr(0), None)
            torch.cuda.synchronize()
            got = out.get(0, np.float32 if out_dt == oracle.F32 else np.uint16)
            _cmp_reduce(got, want, out_dt)
            out.check_guards()
            if G > 8:
                break                      # one pass is enough for the long ones
    finally:
        fcdp.fcdp_tuning_set("reduce_phased", before)
    arena.check_guards()


@pytest.mark.parametrize("G,in_dt,out_dt", [(8, oracle.F32, oracle.F32), (16, oracle.F32, oracle.BF16),
                                            (24, oracle.BF16, oracle.BF16), (8, oracle.BF16, oracle.F32)])
def test_reduce_phased_both_wave_shapes(G, in_dt, out_dt):
    """The phased kernel is built in two shapes (one wave per SIMD holding 104
    steps, two waves holding 52); with full load groups either can run: both
    give the oracle's bits, over one phase and over two."""
    for count in (4194304 + 64 * 4 * 5 + 3, 27262976 + 70003):
        if in_dt == oracle.BF16 and count < 8388608:
            count *= 2                       # bf16 steps are 512 elements: stay above the two-wave threshold
        g = synth.rng(0, 2900 + G, synth.KIND_GRAD, count % 1000)
        parts = []
        for r in range(G):
            x = g.standard_normal(count, dtype=np.float32) * np.float32(1e-3)
            parts.append(x if in_dt == oracle.F32 else synth.to_bf16_bits(x))
        want = oracle.reduce(parts, 0, count, out_dt)
        d_parts = [to_dev(p) for p in parts]
        out = Arena([count * (4 if out_dt == oracle.F32 else 2)])
        before = (fcdp.fcdp_tuning_get("reduce_phased"), fcdp.fcdp_tuning_get("reduce_phase_waves"))
        try:
            fcdp.fcdp_tuning_set("reduce_phased", 1)
            for waves in (1, 2):
                fcdp.fcdp_tuning_set("reduce_phase_waves", waves)
                out.buf.fill_(0xC3)
                fcdp.fcdp_reduce_grad_shard(d_parts, G, 0, count, in_dt, out_dt, out.ptr(0), None)
                torch.cuda.synchronize()
                assert fcdp.fcdp_tuning_get("last_reduce_shape") == waves   # the shape asked for did run
                _cmp_reduce(out.get(0, np.float32 if out_dt == oracle.F32 else np.uint16), want, out_dt)
                out.check_guards()
        finally:
            fcdp.fcdp_tuning_set("reduce_phased", before[0])
            fcdp.fcdp_tuning_set("reduce_phase_waves", before[1])
        del d_parts
        if G > 8:
            break                            # the long case once is enough


FULL_LAUNCH = 1024 * 104 * 256   # elements one phased launch holds on a 256-CU part
RULE_CASES = [  # G, in, out, count -> waves per SIMD of the (first) phased launch, 0 = one tile per workgroup
    (1, oracle.F32, oracle.F32, 20000000, 0), (2, oracle.BF16, oracle.BF16, 20000000, 0),
    (3, oracle.F32, oracle.F32, 20000000, 2), (3, oracle.BF16, oracle.BF16, 20000000, 2),
    (3, oracle.F32, oracle.BF16, 20000000, 0), (4, oracle.BF16, oracle.F32, 20000000, 0),
    (5, oracle.F32, oracle.BF16, 20000000, 2), (6, oracle.BF16, oracle.F32, 20000000, 0),
    (8, oracle.F32, oracle.F32, 20000000, 1), (8, oracle.F32, oracle.BF16, 20000000, 1),
    (8, oracle.BF16, oracle.F32, 20000000, 1), (8, oracle.BF16, oracle.BF16, 20000000, 2),
    (12, oracle.BF16, oracle.F32, 20000000, 2),
    (16, oracle.BF16, oracle.BF16, 20000000, 1), (16, oracle.F32, oracle.BF16, 20000000, 1),
    # by length: the one-wave shape from 0.7 of a full launch on; below that two waves per SIMD
    # for G >= 12 and one tile per workgroup for G = 8; below 0.46 one tile per workgroup
    (8, oracle.F32, oracle.F32, int(0.55 * FULL_LAUNCH), 0), (16, oracle.BF16, oracle.BF16, int(0.55 * FULL_LAUNCH), 2),
    (32, oracle.F32, oracle.BF16, int(0.50 * FULL_LAUNCH), 2), (12, oracle.F32, oracle.F32, int(0.50 * FULL_LAUNCH), 2),
    (16, oracle.F32, oracle.F32, int(0.40 * FULL_LAUNCH), 0), (12, oracle.F32, oracle.F32, int(0.40 * FULL_LAUNCH), 0),
    # beyond one launch: full launches, then the rest judged by its own length
    (8, oracle.F32, oracle.F32, int(1.05 * FULL_LAUNCH), 1), (8, oracle.F32, oracle.F32, int(1.80 * FULL_LAUNCH), 1),
]


@pytest.mark.parametrize("G,in_dt,out_dt,count,shape", RULE_CASES)
def test_reduce_rule_picks_the_documented_shape(G, in_dt, out_dt, count, shape):
    """Left to its rule (the default), the reduce launches the kernel shape the
    header documents for this rank count, type pair and length."""
    if torch.cuda.get_device_properties(0).multi_processor_count != 256:
        pytest.skip("the lengths here are fractions of a launch on a 256-CU part")
    assert fcdp.fcdp_tuning_get("reduce_phased") == 2 and fcdp.fcdp_tuning_get("reduce_phase_waves") == 0
    ies = 4 if in_dt == oracle.F32 else 2
    buf = torch.zeros(count * ies, dtype=torch.uint8, device="cuda")   # every rank reads the same zeros
    out = torch.empty(count * 4, dtype=torch.uint8, device="cuda")
    ptrs = [buf.data_ptr()] * G
    fcdp.fcdp_reduce_grad_shard(ptrs, G, 0, count, in_dt, out_dt, out.data_ptr(), None)
    torch.cuda.synchronize()
    assert fcdp.fcdp_tuning_get("last_reduce_shape") == shape
    assert not bool(out[:count * (4 if out_dt == oracle.F32 else 2)].view(torch.int16).bitwise_and(0x7fff).any())  # sums of zeros


def test_reduce_phased_specials_in_place_and_both_kernels_agree():
    """Through the phased kernel: Inf, NaN, signed zeros, denormals and
    order-sensitive columns give the oracle's bits; rank 1 reduces in place
    into its own slice; and the two kernels give the same bits."""
    G, n = 6, 4194304 + 1028
    specials = np.array([0x00000000, 0x80000000, 0x00000001, 0x80000001, 0x007FFFFF,
                         0x00800000, 0x7F7FFFFF, 0xFF7FFFFF, 0x7F800000, 0xFF800000,
                         0x7FC00000, 0x3F800000, 0xBF800000, 0x4B800000, 0x4B800001,
                         0x33800000, 0x4CBEBC20, 0xCCBEBC20], dtype=np.uint32)
    g = synth.rng(0, 78, synth.KIND_MISC)
    parts = [specials[g.integers(0, specials.size, size=n)].view(np.float32).copy() for _ in range(G)]
    parts[0][:2] = [2.0 ** 24, 1e8]
    parts[1][:2] = [1.0, 1.0]
    parts[2][:2] = [1.0, -1e8]
    for r in range(3, G):
        parts[r][:2] = 0.0
    for r in range(G):
        parts[r][2] = -0.0
    before = fcdp.fcdp_tuning_get("reduce_phased")
    try:
        results = {}
        for knob in (0, 1):
            fcdp.fcdp_tuning_set("reduce_phased", knob)
            for out_dt in (oracle.F32, oracle.BF16):
                with np.errstate(all="ignore"):
                    want = oracle.reduce(parts, 0, n, out_dt)
                arena = Arena([n * 4] * G)
                for r in range(G):
                    arena.fill(r, parts[r])
                out = Arena([n * (4 if out_dt == oracle.F32 else 2)])
                fcdp.fcdp_reduce_grad_shard(arena.ptrs(), G, 0, n, fcdp.F32, out_dt, out.ptr(0), None)
                torch.cuda.synchronize()
                got = out.get(0, np.float32 if out_dt == oracle.F32 else np.uint16)
                _cmp_reduce(got, want, out_dt)
                results[(knob, out_dt)] = got.copy()
                if out_dt == oracle.F32:
                    assert got[0] == np.float32(2.0 ** 24) and got[1] == 0.0
                    assert got.view(np.uint32)[2] == 0x80000000
                    # in place: the sum lands in rank 1's own buffer
                    fcdp.fcdp_reduce_grad_shard(arena.ptrs(), G, 0, n, fcdp.F32, fcdp.F32, arena.ptr(1), None)
                    torch.cuda.synchronize()
                    _cmp_reduce(arena.get(1, np.float32), want, out_dt)
                    arena.check_guards()
        for out_dt in (oracle.F32, oracle.BF16):
            a, b = results[(0, out_dt)], results[(1, out_dt)]
            if out_dt == oracle.F32:
                a, b = a.view(np.uint32), b.view(np.uint32)
                nan = np.isnan(results[(0, out_dt)])
                assert np.array_equal(a[~nan], b[~nan])
            else:
                nan = ((a & 0x7F80) == 0x7F80) & ((a & 0x7F) != 0)   # payloads may differ
                assert np.array_equal(a[~nan], b[~nan])
    finally:
        fcdp.fcdp_tuning_set("reduce_phased", before)


@pytest.mark.parametrize("G,tiles,out_dt", [(1, 3, oracle.F32), (5, 17, oracle.F32), (8, 64, oracle.BF16),
                                            (19, 9, oracle.F32), (32, 33, oracle.BF16), (64, 5, oracle.F32)])
def test_reduce_calibration_stream_is_the_same_sum(G, tiles, out_dt):
    """The measurement probe fcdp_probe_reduce_stream sums, per 1024-element
    tile, the G consecutive sub-tiles of one buffer in order: against the
    oracle's rank-order sum of the G de-interleaved partials."""
    g = synth.rng(0, 600 + G, synth.KIND_GRAD, tiles)
    src = (g.standard_normal((tiles, G, 1024), dtype=np.float32) * np.float32(1e-3))
    parts = [np.ascontiguousarray(src[:, r, :]).reshape(-1) for r in range(G)]
    count = tiles * 1024
    want = oracle.reduce(parts, 0, count, out_dt)
    d_src = to_dev(src)
    out = Arena([count * (4 if out_dt == oracle.F32 else 2)])
    fcdp.fcdp_probe_reduce_stream(out.ptr(0), d_src, G, count, out_dt, None)
    torch.cuda.synchronize()
    _cmp_reduce(out.get(0, np.float32 if out_dt == oracle.F32 else np.uint16), want, out_dt)
    out.check_guards()
    with pytest.raises(fcdp.FcdpError):
        fcdp.fcdp_probe_reduce_stream(out.ptr(0), d_src, G, count - 1, out_dt, None)


PACK_CASES = [
    ("lora_like", [4096, 160, 160, 4096, 160, 160, 9000, 64], [0, 1, 1, 0, 1, 1, 0, 0], 8, 2),
    ("odd", [1001, 3, 777, 0, 12345, 1], [1, 0, 1, 1, 0, 1], 3, 2),
    ("all", [500, 700], [1, 1], 4, 2),
    ("none", [500, 700], [0, 0], 4, 2),
    ("four_byte", [333, 5000, 77], [0, 1, 1], 2, 4),
    ("big_runs", [200000, 70000, 300001, 65536], [1, 0, 1, 1], 5, 2),
]


@pytest.mark.parametrize("name,sizes,tr,G,esz", PACK_CASES, ids=[c[0] for c in PACK_CASES])
def test_pack_unpack_parity(name, sizes, tr, G, esz):
    dt = np.uint16 if esz == 2 else np.uint32
    tensors = _rand_tensors(len(sizes) + 50, sizes, dt)
    flat = oracle.flatten(tensors, G)
    want_packed = oracle.pack(flat, sizes, tr, G)
    L = fcdp.fcdp_layout_build(sizes, tr, G, esz)
    assert L.packed_numel == want_packed.size
    assert L.trainable_numel == sum(k for k, f in zip(sizes, tr) if f)
    fa = Arena([flat.size * esz])
    fa.fill(0, flat)
    pa = Arena([max(want_packed.size, 0) * esz])
    fcdp.fcdp_pack_trainable(L, fa.ptr(0), pa.ptr(0), None)
    torch.cuda.synchronize()
    assert np.array_equal(pa.get(0, dt), want_packed)
    pa.check_guards()
    # unpack new values into a different flat image: frozen bytes untouched
    newp = _rand_tensors(99, [want_packed.size], dt)[0]
    base = _rand_tensors(98, [flat.size], dt)[0]
    want_flat = base.copy()
    oracle.unpack(newp, want_flat, sizes, tr)
    pa.fill(0, newp)
    fb = Arena([flat.size * esz])
    fb.fill(0, base)
    fcdp.fcdp_unpack_trainable(L, pa.ptr(0), fb.ptr(0), None)
    torch.cuda.synchronize()
    assert np.array_equal(fb.get(0, dt), want_flat)
    fb.check_guards()


def test_unpack_refreshes_mapped_host_cache():
    """Unpack straight into the device alias of the host cache refreshes H for
    the trainable parameters only (Alg. 1: only W_t is dirty after a step)."""
    sizes, tr, G = [4096, 128, 128, 8192, 64], [0, 1, 1, 0, 0], 4
    tensors = _rand_tensors(5, sizes, np.uint16)
    flat = oracle.flatten(tensors, G)
    L = fcdp.fcdp_layout_build(sizes, tr, G, 2)
    H = fcdp.fcdp_host_cache_alloc(flat.size * 2)
    H.numpy(np.uint16, flat.size)[:] = flat
    newp = _rand_tensors(6, [L.packed_numel], np.uint16)[0]
    want = flat.copy()
    oracle.unpack(newp, want, sizes, tr)
    d = to_dev(newp)
    fcdp.fcdp_unpack_trainable(L, d, H.dev, None)
    torch.cuda.synchronize()
    assert np.array_equal(H.numpy(np.uint16, flat.size), want)
    H.free()


def test_double_buffered_backward_sweep():
    """Several layers with distinct contents through two staging buffers, no
    host synchronisation between layers: every layer's tensors must be its
    own (a missing wait would show another layer's bytes)."""
    sizes = [3 * 1024 * 1024 + 8, 4096, 5 * 1024 * 1024, 1000001]
    G, esz, nl = 4, 2, 6
    L = fcdp.fcdp_layout_build(sizes, None, G, esz)
    Np = L.padded_numel
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    caches, wants = [], []
    for l in range(nl):
        tensors = _rand_tensors(700 + l, sizes, np.uint16)
        flat = oracle.flatten(tensors, G)
        H = fcdp.fcdp_host_cache_alloc(Np * esz)
        H.numpy(np.uint16, Np)[:] = flat
        caches.append(H)
        wants.append(oracle.materialize_from_flat(flat, sizes))
    staging = [Arena([Np * esz]), Arena([Np * esz])]
    outs = [Arena([k * esz for k in sizes]) for _ in range(nl)]
    torch.cuda.synchronize()
    for l in range(nl - 1, -1, -1):
        fcdp.fcdp_materialize_layer(L, fcdp.SRC_HOST_DMA, None, caches[l],
                                    staging[l % 2].ptr(0), outs[l].ptrs(), False, compute, copy)
    torch.cuda.synchronize()
    for l in range(nl):
        for t in range(len(sizes)):
            assert np.array_equal(outs[l].get(t, np.uint16), wants[l][t]), (l, t)
        outs[l].check_guards()
    for H in caches:
        H.free()


def test_tuning_variants_same_bytes():
    """Every launch shape gives the same bytes (results do not depend on the
    block size, the unroll depth, the grid cap or the access hints)."""
    sizes = [300001, 7, 65537, 131075]
    G = 3
    tensors = _rand_tensors(1, sizes, np.uint16)
    flat = oracle.flatten(tensors, G)
    shards = oracle.split(flat, G)
    parts = [synth.grad_partial_f32(synth.CONFIGS["gpt2_small_g4"], 1, r, 200003) for r in range(5)]
    want_r = oracle.reduce(parts, 3, 200000, oracle.F32)
    pa = Arena([200003 * 4] * 5)
    for r in range(5):
        pa.fill(r, parts[r])
    defaults = {k: fcdp.fcdp_tuning_get(k) for k in
                ("copy_chunk_bytes", "copy_block", "copy_unroll", "copy_wg_per_cu", "copy_nt",
                 "reduce_block")}
    try:
        for chunk, block, unroll, wg, nt in [(4096, 64, 1, 0, 0), (16384, 128, 2, 2, 1),
                                             (65536, 256, 4, 0, 1), (262144, 512, 8, 4, 0),
                                             (1 << 20, 1024, 8, 1, 1)]:
            fcdp.fcdp_tuning_set("copy_chunk_bytes", chunk)
            fcdp.fcdp_tuning_set("copy_block", block)
            fcdp.fcdp_tuning_set("copy_unroll", unroll)
            fcdp.fcdp_tuning_set("copy_wg_per_cu", wg)
            fcdp.fcdp_tuning_set("copy_nt", nt)
            L = fcdp.fcdp_layout_build(sizes, None, G, 2)
            sh = Arena([L.shard_numel * 2] * G)
            for r in range(G):
                sh.fill(r, shards[r])
            out = Arena([k * 2 for k in sizes])
            fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, sh.ptrs(), None, None, out.ptrs())
            torch.cuda.synchronize()
            for t in range(len(sizes)):
                assert np.array_equal(out.get(t, np.uint16), tensors[t])
            out.check_guards()
        for block in (64, 128, 256):
            fcdp.fcdp_tuning_set("reduce_block", block)
            out = Arena([200000 * 4])
            fcdp.fcdp_reduce_grad_shard(pa.ptrs(), 5, 3, 200000, fcdp.F32, fcdp.F32, out.ptr(0))
            torch.cuda.synchronize()
            assert np.array_equal(out.get(0, np.float32).view(np.uint32), want_r.view(np.uint32))
            out.check_guards()
    finally:
        for k, v in defaults.items():
            fcdp.fcdp_tuning_set(k, v)


def test_every_host_link_path_rejects_pageable_memory():
    """Sec. 4.4 wants the cache in pinned buffers: a numpy array (pageable)
    as host_cache is FCDP_ENOTPINNED on every path that crosses the host
    link, before anything is enqueued; pinned memory that is not from
    fcdp_host_cache_alloc (torch's pin_memory) is accepted by the DMA paths
    and gives the oracle's bytes."""
    sizes, G = [5000, 3, 70001], 4
    tensors = _rand_tensors(9, sizes, np.uint16)
    flat = oracle.flatten(tensors, G)
    shards = oracle.split(flat, G)
    L = fcdp.fcdp_layout_build(sizes, None, G, 2)
    L.prepare()
    Np = L.padded_numel
    sh = Arena([L.shard_numel * 2] * G)
    for r in range(G):
        sh.fill(r, shards[r])
    out = Arena([k * 2 for k in sizes])
    staging = Arena([Np * 2])
    pageable = np.zeros(Np, dtype=np.uint16)
    pageable[:] = flat
    hp = pageable.ctypes.data
    assert hp % 16 == 0
    sentinel_before = out.buf.clone()
    calls = {
        "host_dma": lambda h: fcdp.fcdp_materialize_layer(L, fcdp.SRC_HOST_DMA, None, h, staging.ptr(0), out.ptrs()),
        "host_scatter_dma": lambda h: fcdp.fcdp_materialize_layer(L, fcdp.SRC_HOST_SCATTER_DMA, None, h, None, out.ptrs()),
        "host_zerocopy": lambda h: fcdp.fcdp_materialize_layer(L, fcdp.SRC_HOST_ZEROCOPY, None, h, None, out.ptrs()),
        "static": lambda h: fcdp.fcdp_materialize_layer_static(L, h, out.ptrs()),
        "store_dma": lambda h: fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, sh.ptrs(), h, None, out.ptrs(),
                                                           fcdp.STORE_DMA),
        "store_zerocopy": lambda h: fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, sh.ptrs(), h, None,
                                                                out.ptrs(), fcdp.STORE_ZEROCOPY),
        "cache_store_dma": lambda h: fcdp.fcdp_cache_store(L, sh.ptrs(), h, fcdp.STORE_DMA),
        "cache_store_zerocopy": lambda h: fcdp.fcdp_cache_store(L, sh.ptrs(), h, fcdp.STORE_ZEROCOPY),
        "node_slice_store": lambda h: fcdp.fcdp_cache_store_node_slice(L, 1, 2, sh.ptrs(), h),
        "node_slice_fetch": lambda h: fcdp.fcdp_materialize_layer_node_slice(L, 1, 2, sh.ptrs(), h, staging.ptr(0),
                                                                             out.ptrs()),
    }
    for name, call in calls.items():
        with pytest.raises(fcdp.FcdpError) as e:
            call(hp)
        assert e.value.name == "FCDP_ENOTPINNED", name
    torch.cuda.synchronize()
    assert torch.equal(out.buf, sentinel_before), "a refused call wrote to the tensors"
    # pinned memory from another allocator: fine for the DMA paths
    pinned = torch.empty(Np, dtype=torch.int16).pin_memory()
    fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, sh.ptrs(), pinned.data_ptr(), None, out.ptrs(),
                                fcdp.STORE_DMA)
    torch.cuda.synchronize()
    assert np.array_equal(pinned.numpy().view(np.uint16), flat)
    for name in ("host_dma", "host_scatter_dma", "static"):
        out.buf.fill_(0xC3)
        calls[name](pinned.data_ptr())
        torch.cuda.synchronize()
        for t in range(len(sizes)):
            assert np.array_equal(out.get(t, np.uint16), tensors[t]), name
        out.check_guards()


def test_zero_copy_rejects_unpinned_memory():
    sizes, G = [1024], 2
    L = fcdp.fcdp_layout_build(sizes, None, G, 2)
    out = Arena([2048])
    host = np.zeros(L.padded_numel, dtype=np.uint16)
    with pytest.raises(fcdp.FcdpError) as e:
        fcdp.fcdp_materialize_layer(L, fcdp.SRC_HOST_ZEROCOPY, None, host.ctypes.data, None, out.ptrs())
    assert e.value.name == "FCDP_ENOTPINNED"
    # the failed call left no sticky error behind: a good call still works
    sh = Arena([L.shard_numel * 2] * G)
    fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, sh.ptrs(), None, None, out.ptrs())
    torch.cuda.synchronize()


def test_probe_copy():
    n = 3 * 1024 * 1024 + 10
    x = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda")
    y = torch.zeros_like(x)
    fcdp.fcdp_probe_copy(y, x, n, None)
    torch.cuda.synchronize()
    assert torch.equal(x, y)


def test_kernel_timing_hooks():
    """Timed dispatches are counted per kind and report plausible durations."""
    n = 1 << 22
    x = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda")
    y = torch.zeros_like(x)
    parts = [torch.ones(n // 4, dtype=torch.float32, device="cuda") for _ in range(3)]
    out = torch.zeros(n // 4, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    fcdp.fcdp_timing_enable(8)
    try:
        for _ in range(3):
            fcdp.fcdp_probe_copy(y, x, n, None)
        fcdp.fcdp_reduce_grad_shard(parts, 3, 0, n // 4, fcdp.F32, fcdp.F32, out, None)
        torch.cuda.synchronize()
        cnt, ms = fcdp.fcdp_timing_collect(fcdp.KERNEL_PROBE_COPY)
        assert cnt == 3 and 0.0 < ms < 50.0
        cnt, ms = fcdp.fcdp_timing_collect(fcdp.KERNEL_REDUCE)
        assert cnt == 1 and 0.0 < ms < 50.0
        assert fcdp.fcdp_timing_collect(fcdp.KERNEL_PACK) == (0, 0.0)
        # the pool is bounded: launches beyond the capacity are simply not timed
        for _ in range(12):
            fcdp.fcdp_probe_copy(y, x, n, None)
        torch.cuda.synchronize()
        cnt, ms = fcdp.fcdp_timing_collect(fcdp.KERNEL_PROBE_COPY)
        assert cnt == 8
    finally:
        fcdp.fcdp_timing_enable(0)
    assert torch.equal(x, y) and float(out[0]) == 3.0


TRAINABLE_REDUCE_CASES = [
    ("lora_like", [4096, 160, 160, 4096, 160, 160, 9000, 64], [0, 1, 1, 0, 1, 1, 0, 0], 8, oracle.F32, oracle.F32),
    ("odd", [1001, 3, 777, 0, 12345, 1], [1, 0, 1, 1, 0, 1], 3, oracle.F32, oracle.F32),
    ("odd_bf16_out", [1001, 3, 777, 0, 12345, 1], [1, 0, 1, 1, 0, 1], 3, oracle.F32, oracle.BF16),
    ("bf16_in", [333, 5001, 77, 2050], [0, 1, 1, 1], 4, oracle.BF16, oracle.F32),
    ("bf16_in_out", [333, 5001, 77, 2050], [1, 1, 0, 1], 2, oracle.BF16, oracle.BF16),
    ("big_runs", [200000, 70000, 300001, 65536], [1, 0, 1, 1], 5, oracle.F32, oracle.F32),
    ("none_trainable", [500, 700], [0, 0], 4, oracle.F32, oracle.F32),
    ("all_trainable_one_rank", [500, 700, 9], [1, 1, 1], 1, oracle.F32, oracle.BF16),
    ("many_runs", [(37 * i) % 90 + 1 for i in range(150)], [i % 2 for i in range(150)], 2, oracle.F32, oracle.F32),
]


@pytest.mark.parametrize("name,sizes,tr,G,in_dt,out_dt", TRAINABLE_REDUCE_CASES,
                         ids=[c[0] for c in TRAINABLE_REDUCE_CASES])
def test_reduce_trainable_shard_parity(name, sizes, tr, G, in_dt, out_dt):
    """Pack and reduce in one launch, for every rank, against the oracle's
    pack followed by its rank-order reduce."""
    L = fcdp.fcdp_layout_build(sizes, tr, G, 2)
    Np = L.padded_numel
    g = synth.rng(0, 1200 + G, synth.KIND_GRAD, len(sizes))
    parts = []
    for r in range(G):
        x = g.standard_normal(Np, dtype=np.float32) * np.float32(10.0 ** int(g.integers(-4, 2)))
        parts.append(x if in_dt == oracle.F32 else synth.to_bf16_bits(x))
    ies = 4 if in_dt == oracle.F32 else 2
    oes = 4 if out_dt == oracle.F32 else 2
    arena = Arena([Np * ies] * G)
    for r in range(G):
        arena.fill(r, parts[r])
    Sp = L.packed_numel // G
    for rank in range(G):
        # the oracle packs each rank's gradient, then sums the packed slices
        want = oracle.reduce_trainable(parts, sizes, tr, G, rank, out_dt)
        assert want.size == Sp
        out = Arena([Sp * oes])
        fcdp.fcdp_reduce_trainable_shard(L, arena.ptrs(), rank, in_dt, out_dt, out.ptr(0), None)
        torch.cuda.synchronize()
        got = out.get(0, np.float32 if out_dt == oracle.F32 else np.uint16)
        _cmp_reduce(got, want, out_dt)
        out.check_guards()
    arena.check_guards()


SCALED_CASES = [
    # G, count, e0, in, out, scale
    (8, 300007, 0, oracle.F32, oracle.F32, 1.0 / 8),
    (8, 300007, 0, oracle.F32, oracle.BF16, 1.0 / 8),
    (3, 70001, 5, oracle.F32, oracle.F32, 1.0 / 3),
    (7, 33333, 3, oracle.F32, oracle.BF16, 1.0 / 7),
    (17, 40000, 7, oracle.F32, oracle.F32, 1.0 / 17),
    (5, 50001, 0, oracle.BF16, oracle.BF16, 0.2),
    (32, 9999, 5, oracle.BF16, oracle.F32, 1.0 / (32 * 1024.0)),
    (4, 4099, 1, oracle.F32, oracle.F32, -3.5),
    (2, 1003, 0, oracle.F32, oracle.F32, 0.0),
    (6, 3, 0, oracle.F32, oracle.F32, 1.0 / 6),
]


@pytest.mark.parametrize("G,count,e0,in_dt,out_dt,scale", SCALED_CASES)
def test_scaled_reduce_parity(G, count, e0, in_dt, out_dt, scale):
    """Sum in rank order, then one multiplication by the given float."""
    scale = float(np.float32(scale))
    g = synth.rng(0, 1700 + G, synth.KIND_GRAD, count % 1000)
    total = e0 + count + 5
    parts = []
    for r in range(G):
        x = g.standard_normal(total, dtype=np.float32) * np.float32(10.0 ** int(g.integers(-5, 2)))
        parts.append(x if in_dt == oracle.F32 else synth.to_bf16_bits(x))
    want = oracle.reduce(parts, e0, count, out_dt, scale)
    ies = 4 if in_dt == oracle.F32 else 2
    oes = 4 if out_dt == oracle.F32 else 2
    arena = Arena([total * ies] * G)
    for r in range(G):
        arena.fill(r, parts[r])
    out = Arena([count * oes])
    fcdp.fcdp_reduce_grad_shard_scaled(arena.ptrs(), G, e0, count, in_dt, out_dt,
                                       scale, out.ptr(0), None)
    torch.cuda.synchronize()
    got = out.get(0, np.float32 if out_dt == oracle.F32 else np.uint16)
    _cmp_reduce(got, want, out_dt)
    out.check_guards()


def test_scale_one_is_the_plain_sum_and_denormals_survive():
    """scale = 1 gives the unscaled entry point's bits, including denormal
    and negative-zero results; scaling into the denormal range rounds as IEEE
    arithmetic does, with no flush."""
    n = 4096 + 3
    g = synth.rng(0, 1801, synth.KIND_GRAD)
    parts = [g.standard_normal(n, dtype=np.float32) for _ in range(3)]
    for p in parts:
        p[:64] = np.arange(1, 65, dtype=np.uint32).view(np.float32)   # denormals
        p[64:80] = -0.0
    arena = Arena([n * 4] * 3)
    for r in range(3):
        arena.fill(r, parts[r])
    a, b, c = Arena([n * 4]), Arena([n * 4]), Arena([n * 4])
    fcdp.fcdp_reduce_grad_shard(arena.ptrs(), 3, 0, n, fcdp.F32, fcdp.F32, a.ptr(0), None)
    fcdp.fcdp_reduce_grad_shard_scaled(arena.ptrs(), 3, 0, n, fcdp.F32, fcdp.F32, 1.0, b.ptr(0), None)
    tiny = float(np.float32(2.0 ** -130))
    fcdp.fcdp_reduce_grad_shard_scaled(arena.ptrs(), 3, 0, n, fcdp.F32, fcdp.F32, tiny, c.ptr(0), None)
    torch.cuda.synchronize()
    plain = a.get(0, np.uint32)
    assert np.array_equal(plain, b.get(0, np.uint32))
    assert np.array_equal(plain, oracle.reduce(parts, 0, n, oracle.F32).view(np.uint32))
    want = oracle.reduce(parts, 0, n, oracle.F32, tiny)
    assert np.count_nonzero((want != 0) & (np.abs(want) < 2.0 ** -126)) > 100    # denormal results
    assert np.array_equal(c.get(0, np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("name,sizes,tr,G,in_dt,out_dt", TRAINABLE_REDUCE_CASES[:4],
                         ids=[c[0] for c in TRAINABLE_REDUCE_CASES[:4]])
def test_scaled_reduce_trainable_shard_parity(name, sizes, tr, G, in_dt, out_dt):
    """The fused pack + reduce with the mean's scale, every rank."""
    L = fcdp.fcdp_layout_build(sizes, tr, G, 2)
    Np = L.padded_numel
    scale = float(np.float32(-1.0) / np.float32(G))      # a negative scale: the zero tail is -0
    g = synth.rng(0, 1900 + G, synth.KIND_GRAD, len(sizes))
    parts = []
    for r in range(G):
        x = g.standard_normal(Np, dtype=np.float32)
        parts.append(x if in_dt == oracle.F32 else synth.to_bf16_bits(x))
    ies = 4 if in_dt == oracle.F32 else 2
    oes = 4 if out_dt == oracle.F32 else 2
    arena = Arena([Np * ies] * G)
    for r in range(G):
        arena.fill(r, parts[r])
    Sp = L.packed_numel // G
    for rank in range(G):
        want = oracle.reduce_trainable(parts, sizes, tr, G, rank, out_dt, scale=scale)
        out = Arena([Sp * oes])
        fcdp.fcdp_reduce_trainable_shard_scaled(L, arena.ptrs(), rank, in_dt, out_dt,
                                                scale, out.ptr(0), None)
        torch.cuda.synchronize()
        got = out.get(0, np.float32 if out_dt == oracle.F32 else np.uint16)
        _cmp_reduce(got, want, out_dt)
        out.check_guards()


def test_whole_model_layout_many_tensors():
    """One layout over every layer's tensors (more tensors than one launch's
    pointer window): unflatten runs as several launches, pack and unpack as
    one; all against the oracle."""
    layer = [4096, 96, 96, 2048, 64, 64, 7000, 33]
    tr_layer = [0, 1, 1, 0, 1, 1, 0, 0]
    nl, G = 40, 4                               # 320 tensors
    sizes, tr = layer * nl, tr_layer * nl
    tensors = _rand_tensors(31, sizes, np.uint16)
    flat = oracle.flatten(tensors, G)
    shards = oracle.split(flat, G)
    L = fcdp.fcdp_layout_build(sizes, tr, G, 2)
    sh = Arena([L.shard_numel * 2] * G)
    for r in range(G):
        sh.fill(r, shards[r])
    out = Arena([k * 2 for k in sizes])
    fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, sh.ptrs(), None, None, out.ptrs())
    torch.cuda.synchronize()
    for t in range(len(sizes)):
        assert np.array_equal(out.get(t, np.uint16), tensors[t]), t
    out.check_guards()
    fa = Arena([flat.size * 2]); fa.fill(0, flat)
    pa = Arena([L.packed_numel * 2])
    fcdp.fcdp_pack_trainable(L, fa.ptr(0), pa.ptr(0), None)
    torch.cuda.synchronize()
    assert np.array_equal(pa.get(0, np.uint16), oracle.pack(flat, sizes, tr, G))
    pa.check_guards()
    back = Arena([L.shard_numel * 2] * G)
    fcdp.fcdp_flatten_to_shards(L, out.ptrs(), back.ptrs(), None)
    torch.cuda.synchronize()
    for r in range(G):
        assert np.array_equal(back.get(r, np.uint16), shards[r])


def test_random_layouts_end_to_end():
    """Forty seeded random layers (tensor counts 1..40, sizes 0..400k, every G
    class, both element sizes, random trainable masks) through every byte
    mover: unflatten + store, the three host fetches, flatten, pack, unpack."""
    g = synth.rng(0, 4242, synth.KIND_MISC, 5)
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    for case in range(40):
        T = int(g.integers(1, 41))
        G = int(g.choice([1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64]))
        esz = int(g.choice([2, 4]))
        sizes = synth.random_layer(9000 + case, T=T, max_numel=int(g.choice([300, 5000, 400000])))
        tr = [int(v) for v in g.integers(0, 2, size=T)]
        dt = np.uint16 if esz == 2 else np.uint32
        tensors = _rand_tensors(5000 + case, sizes, dt)
        flat = oracle.flatten(tensors, G)
        shards = oracle.split(flat, G)
        L = fcdp.fcdp_layout_build(sizes, tr, G, esz)
        S, Np, Pn = L.shard_numel, L.padded_numel, L.packed_numel
        tag = (case, T, G, esz)
        sh = Arena([S * esz] * G)
        for r in range(G):
            sh.fill(r, shards[r])
        H = fcdp.fcdp_host_cache_alloc(max(Np * esz, 16))
        H.numpy(np.uint8)[:] = 0x5A
        out = Arena([k * esz for k in sizes])
        torch.cuda.synchronize()
        fcdp.fcdp_materialize_layer(L, fcdp.SRC_DEVICE_SHARDS, sh.ptrs(), H, None, out.ptrs(),
                                    fcdp.STORE_DMA if case % 2 else fcdp.STORE_ZEROCOPY, compute, copy)
        torch.cuda.synchronize()
        for t in range(T):
            assert np.array_equal(out.get(t, dt), tensors[t]), tag + ("shards", t)
        out.check_guards()
        assert np.array_equal(H.numpy(dt, Np), flat), tag + ("store",)
        for mode in (fcdp.SRC_HOST_DMA, fcdp.SRC_HOST_ZEROCOPY, fcdp.SRC_HOST_SCATTER_DMA):
            o2 = Arena([k * esz for k in sizes])
            stg = Arena([max(Np * esz, 16)])
            torch.cuda.synchronize()
            fcdp.fcdp_materialize_layer(L, mode, None, H, stg.ptr(0), o2.ptrs(), fcdp.STORE_NONE,
                                        compute, copy)
            torch.cuda.synchronize()
            for t in range(T):
                assert np.array_equal(o2.get(t, dt), tensors[t]), tag + (mode, t)
            o2.check_guards()
            stg.check_guards()
        back = Arena([S * esz] * G)
        fcdp.fcdp_flatten_to_shards(L, out.ptrs(), back.ptrs(), compute)
        fl = Arena([max(Np * esz, 16)])
        fl.buf[fl.ranges[0][0]:fl.ranges[0][0] + Np * esz] = torch.from_numpy(flat.view(np.uint8).copy()).cuda()
        pk = Arena([max(Pn * esz, 16)])
        torch.cuda.synchronize()
        fcdp.fcdp_pack_trainable(L, fl.ptr(0), pk.ptr(0), compute)
        torch.cuda.synchronize()
        for r in range(G):
            assert np.array_equal(back.get(r, dt), shards[r]), tag + ("flatten", r)
        back.check_guards()
        assert np.array_equal(pk.get(0, dt)[:Pn], oracle.pack(flat, sizes, tr, G)), tag + ("pack",)
        pk.check_guards()
        newp = _rand_tensors(7000 + case, [Pn], dt)[0]
        want = flat.copy()
        oracle.unpack(newp, want, sizes, tr)
        if Pn:
            pk.buf[pk.ranges[0][0]:pk.ranges[0][0] + Pn * esz] = torch.from_numpy(newp.view(np.uint8).copy()).cuda()
        torch.cuda.synchronize()
        fcdp.fcdp_unpack_trainable(L, pk.ptr(0), fl.ptr(0), compute)
        torch.cuda.synchronize()
        assert np.array_equal(fl.get(0, dt)[:Np], want), tag + ("unpack",)
        fl.check_guards()
        H.free()
