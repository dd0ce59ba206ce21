#!/usr/bin/env python3
"""Benchmark of the FCDP per-layer hot path on one MI355X.

One step = one pass of the whole path over a Llama-2-7B-shaped stack (32
layers, G = 8 shards per layer, bf16 parameters, fp32 gradient partials):

  forward, layer 0..L-1   unflatten the G gathered shards into the per-tensor
                          parameters (kernel, HBM-bound) and store the flat
                          image to the pinned host cache (D2H DMA, side stream)
  backward, layer L-1..0  fetch the layer from the host cache (H2D DMA through
                          two staging buffers, or the zero-copy kernel),
                          unflatten it, and reduce the G partial gradient
                          slices into this rank's fp32 shard (kernel)
  PEFT leg                pack the LoRA parameters out of the flat buffer,
                          reduce their G packed gradient partials, unpack

Inputs are synthetic and seeded, already resident in HBM / pinned memory when
the timed region starts.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
LINK_PEAK_GBPS = 63.0           # PCIe Gen5 x16 per direction, 128b/130b

# HBM bytes per unflatten launch measured with rocprofv3 --pmc (FETCH_SIZE
# x 1.9998, WRITE_SIZE x 1.0, the factors the same counters show for the
# plain copy of known size); profiles/unflatten_reduce_llama7b_g8_hbm_traffic.md
MEASURED_TRAFFIC = {"llama7b_g8": 822.2e6, "llama7b_lora_g8": 823.3e6,
                    "llama13b_g16": 1288.7e6, "llama70b_g32": 3476.0e6}
MEASURED_TRAFFIC_REDUCE = {"llama7b_g8": 910.7e6, "llama7b_lora_g8": 911.9e6,
                           "llama13b_g16": 1348.1e6, "llama70b_g32": 3529.5e6}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="llama7b_g8")
    ap.add_argument("--layers", type=int, default=0, help="0 = the config's layer count")
    ap.add_argument("--fetch", choices=["dma", "zerocopy", "scatter"], default="dma")
    ap.add_argument("--store", choices=["dma", "zerocopy"], default="dma")
    ap.add_argument("--tau", type=float, default=0.0,
                    help="adaptive GPU caching threshold (Sec. 4.4); 0 = offload every layer")
    ap.add_argument("--no-pretouch", action="store_true")
    ap.add_argument("--copies-in-flight", type=int, default=-1, help="-1 = the library default")
    ap.add_argument("--timed-dispatches", type=int, default=-1,
                    help="how many kernel dispatches carry timing events (-1 = all of the timed steps)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-small-leg", action="store_true",
                    help="skip the launch-bound GPT-2-small leg (eager against a HIP graph)")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--cpu-sample-layers", type=int, default=16)
    ap.add_argument("--cpu-threads", type=int, default=8,
                    help="threads of the all-threads oracle leg (one layer each, ~1.3 GB of host memory per thread)")
    ap.add_argument("--probe-gib", type=int, default=2, help="size of the host-link probe copy")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no "
              "second device); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2602_06499_amd as fcdp
    from paper_2602_06499_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS[args.config]
    L = args.layers or cfg.layers
    G, T = cfg.G, len(cfg.numel)
    if args.copies_in_flight >= 0:
        fcdp.fcdp_tuning_set("max_copies_in_flight", args.copies_in_flight)
    lay = fcdp.fcdp_layout_build(cfg.numel, cfg.trainable, G, 2)
    lay.prepare()
    N, Np, S = lay.numel, lay.padded_numel, lay.shard_numel
    layer_bytes = Np * 2

    def log(msg):
        print("[bench] " + msg, file=sys.stderr, flush=True)

    log("%s: %d layers, N=%d, G=%d, S=%d, %.1f MB/layer" % (cfg.name, L, N, G, S, layer_bytes / 1e6))

    # ---- inputs, resident before timing --------------------------------
    gathered = []        # per layer: the G shards as one gather buffer
    partials = []        # per layer: G fp32 slices of S elements (this rank's slice)
    for l in range(L):
        g = synth.torch_device_generator(dev, cfg.config_id, l, synth.KIND_PARAM)
        w = torch.empty(Np, dtype=torch.bfloat16, device=dev)
        w.normal_(0.0, 0.02, generator=g)
        if Np > N:
            w[N:] = 0
        gathered.append(w)
        g = synth.torch_device_generator(dev, cfg.config_id, l, synth.KIND_GRAD)
        p = torch.empty(G, S, dtype=torch.float32, device=dev)
        p.normal_(0.0, 1e-3, generator=g)
        partials.append(p)
    tensors = [torch.empty(max(k, 1), dtype=torch.bfloat16, device=dev) for k in cfg.numel]
    # adaptive caching: a synthetic activation-memory curve, utilisation rising
    # linearly from 35 % before the first layer to 95 % after the last; a kept
    # layer needs its own tensor set until its backward pass
    state = fcdp.CacheState(L)
    state.set_tau(args.tau)
    total_mem = torch.cuda.get_device_properties(0).total_memory
    util = [0.35 + 0.60 * (l + 1) / L for l in range(L)]
    kept_sets, kept_tensors = {}, {}
    if args.tau > 0:
        for l in range(L):
            if util[l] < args.tau:
                kept_tensors[l] = [torch.empty(max(k, 1), dtype=torch.bfloat16, device=dev) for k in cfg.numel]
                kept_sets[l] = fcdp.pointer_array(kept_tensors[l])
    staging = [torch.empty(Np, dtype=torch.bfloat16, device=dev) for _ in range(2)]
    grad_shard = torch.empty(S, dtype=torch.float32, device=dev)
    t0 = time.time()
    cache = fcdp.fcdp_host_cache_alloc(layer_bytes * L)
    if not args.no_pretouch:
        cache.numpy(np.uint8)[:] = 0        # touch every page before timing
    log("pinned host cache: %.2f GB allocated and touched in %.1f s" % (layer_bytes * L / 1e9, time.time() - t0))
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    host_mode = {"dma": fcdp.SRC_HOST_DMA, "zerocopy": fcdp.SRC_HOST_ZEROCOPY,
                 "scatter": fcdp.SRC_HOST_SCATTER_DMA}[args.fetch]
    store_mode = fcdp.STORE_DMA if args.store == "dma" else fcdp.STORE_ZEROCOPY
    shard_ptrs = [fcdp.pointer_array([w.data_ptr() + r * S * 2 for r in range(G)]) for w in gathered]
    part_ptrs = [fcdp.pointer_array([p.data_ptr() + r * S * 4 for r in range(G)]) for p in partials]
    tensor_ptrs = fcdp.pointer_array(tensors)
    torch.cuda.synchronize()

    def one_step(record):
        """record: None, or a list that collects the sweep events."""
        ev = torch.cuda.Event
        if record is not None:
            e0 = ev(enable_timing=True); e0.record(compute)
        for l in range(L):
            src, _ = state.forward_source(l, 1, host_mode)          # full fine-tuning: always a miss
            tp = kept_sets.get(l, tensor_ptrs)
            if args.tau > 0:
                fcdp.fcdp_materialize_layer(lay, src, shard_ptrs[l], None, None, tp,
                                            fcdp.STORE_NONE, compute, copy)
                # (the layer's forward computation would run here)
                if not state.place(l, int(util[l] * total_mem), total_mem):
                    fcdp.fcdp_cache_store(lay, shard_ptrs[l], cache.host + l * layer_bytes,
                                          store_mode, compute, copy)
            else:
                fcdp.fcdp_materialize_layer(lay, src, shard_ptrs[l],
                                            cache.host + l * layer_bytes, None, tp,
                                            store_mode, compute, copy)
                state.place(l, total_mem, total_mem)
        if record is not None:
            e1 = ev(enable_timing=True); e1.record(copy)
        for l in range(L - 1, -1, -1):
            src = state.backward_source(l, 1, host_mode)
            fcdp.fcdp_materialize_layer(lay, src, None, cache.host + l * layer_bytes,
                                        staging[l % 2], kept_sets.get(l, tensor_ptrs), False,
                                        compute, copy)
            state.release(l)
            fcdp.fcdp_reduce_grad_shard(part_ptrs[l], G, 0, S, fcdp.F32, fcdp.F32,
                                        grad_shard, compute)
        state.optimizer_step()
        if record is not None:
            e2 = ev(enable_timing=True); e2.record(compute)
            record.append((e0, e1, e2))

    for _ in range(args.warmup):
        one_step(None)
    torch.cuda.synchronize()
    # every kernel dispatch of the timed steps carries its own start/stop
    # events (recorded by the library on the stream it launches on)
    fcdp.fcdp_timing_enable(args.steps * L * 3 + 64 if args.timed_dispatches < 0 else args.timed_dispatches)
    fcdp.fcdp_link_bytes(True)
    sweeps = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step(sweeps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps

    link_stored, link_fetched = fcdp.fcdp_link_bytes()
    k1_kind = fcdp.KERNEL_UNFLATTEN
    k1_launches, k1_total = fcdp.fcdp_timing_collect(k1_kind)
    zc_launches, zc_total = fcdp.fcdp_timing_collect(fcdp.KERNEL_UNFLATTEN_ZEROCOPY)
    k3_launches, k3_total = fcdp.fcdp_timing_collect(fcdp.KERNEL_REDUCE)
    fcdp.fcdp_timing_enable(0)
    k1_ms = k1_total / max(k1_launches, 1)
    k3_ms = k3_total / max(k3_launches, 1)
    fwd_ms = sum(e0.elapsed_time(e1) for e0, e1, e2 in sweeps) / args.steps
    bwd_ms = sum(e1.elapsed_time(e2) for e0, e1, e2 in sweeps) / args.steps
    k1_bytes = 4 * N                        # read N*2 + write N*2
    k3_bytes = G * S * 4 + S * 4            # read G fp32 slices + write one
    k1_gbps = k1_bytes / (k1_ms * 1e-3) / 1e9 if k1_ms else 0.0
    k3_gbps = k3_bytes / (k3_ms * 1e-3) / 1e9 if k3_ms else 0.0
    d2h_gbps = link_stored / args.steps / (fwd_ms * 1e-3) / 1e9
    h2d_gbps = link_fetched / args.steps / (bwd_ms * 1e-3) / 1e9
    value = 2 * L * layer_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- self-check outside the timed region ---------------------------
    if not args.no_check:
        off = lay.offsets
        flat0 = gathered[0]
        last = kept_tensors.get(0, tensors)
        for t, k in enumerate(cfg.numel):
            assert torch.equal(last[t][:k], flat0[off[t]:off[t] + k]), "materialized tensor mismatch"
        acc = partials[0][0].clone()
        for r in range(1, G):
            acc = acc + partials[0][r]
        assert torch.equal(acc.view(torch.int32), grad_shard.view(torch.int32)), "gradient shard mismatch"
        if (L - 1) not in kept_sets:
            hc = torch.from_numpy(cache.numpy(np.int16, Np, (L - 1) * layer_bytes))
            assert torch.equal(hc, gathered[L - 1].cpu().view(torch.int16)), "host cache mismatch"

    # ---- host-link probe: one large pinned copy each way ----------------
    probe_bytes = args.probe_gib << 30
    pin = torch.empty(probe_bytes, dtype=torch.uint8, pin_memory=True)
    dbuf = torch.empty(probe_bytes, dtype=torch.uint8, device=dev)
    link = {}
    for name, (dst, src) in (("h2d", (dbuf, pin)), ("d2h", (pin, dbuf))):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        best = 0.0
        for _ in range(2):
            a.record(); dst.copy_(src, non_blocking=True); b.record(); torch.cuda.synchronize()
            best = max(best, probe_bytes / (a.elapsed_time(b) * 1e-3) / 1e9)
        link[name] = best
    del dbuf, pin

    # ---- plain copy reference and the other path variants ---------------
    def time_kernel(fn, reps=10):
        fn(); torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(compute)
        for _ in range(reps):
            fn()
        b.record(compute); torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    ref_dst = torch.empty(Np, dtype=torch.bfloat16, device=dev)
    copy_ms = time_kernel(lambda: fcdp.fcdp_probe_copy(ref_dst, gathered[0], N * 2, compute))
    del ref_dst
    zc_ms = time_kernel(lambda: fcdp.fcdp_materialize_layer(
        lay, fcdp.SRC_HOST_ZEROCOPY, None, cache.host, None, tensors, False, compute, copy), reps=3)
    dma_ms = time_kernel(lambda: fcdp.fcdp_materialize_layer(
        lay, fcdp.SRC_HOST_DMA, None, cache.host, staging[0], tensors, False, compute, copy), reps=3)
    sc_ms = time_kernel(lambda: fcdp.fcdp_materialize_layer(
        lay, fcdp.SRC_HOST_SCATTER_DMA, None, cache.host, None, tensors, False, compute, copy), reps=3)
    bshard = torch.empty(S, dtype=torch.bfloat16, device=dev)
    k3b_ms = time_kernel(lambda: fcdp.fcdp_reduce_grad_shard(
        part_ptrs[0], G, 0, S, fcdp.F32, fcdp.BF16, bshard, compute))

    # bf16 partials (half the read bytes): the first half of each fp32 partial viewed as bf16
    bpart = fcdp.pointer_array([partials[0][r] for r in range(G)])
    k3bb_ms = time_kernel(lambda: fcdp.fcdp_reduce_grad_shard(
        bpart, G, 0, S, fcdp.BF16, fcdp.BF16, bshard, compute))

    # ---- PEFT leg: LoRA r16 on q,v of the same stack ---------------------
    pcfg = synth.CONFIGS["llama7b_lora_g8"]
    play = fcdp.fcdp_layout_build(pcfg.numel, pcfg.trainable, pcfg.G, 2)
    play.prepare()
    pflat = torch.zeros(play.padded_numel, dtype=torch.bfloat16, device=dev)
    ppacked = torch.zeros(play.packed_numel, dtype=torch.bfloat16, device=dev)
    pS = play.packed_numel // pcfg.G
    pgrads = torch.zeros(pcfg.G, pS, dtype=torch.float32, device=dev).normal_(0, 1e-3)
    pg_ptrs = [pgrads.data_ptr() + r * pS * 4 for r in range(pcfg.G)]
    pshard = torch.zeros(pS, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    pack_us = 1e3 * time_kernel(lambda: fcdp.fcdp_pack_trainable(play, pflat, ppacked, compute), reps=50)
    unpack_us = 1e3 * time_kernel(lambda: fcdp.fcdp_unpack_trainable(play, ppacked, pflat, compute), reps=50)
    pred_us = 1e3 * time_kernel(lambda: fcdp.fcdp_reduce_grad_shard(
        pg_ptrs, pcfg.G, 0, pS, fcdp.F32, fcdp.F32, pshard, compute), reps=50)
    # the same from G unpacked flat gradients: G packs + one reduce, against the fused launch
    # (all G flat gradients alias one buffer here: only the launch pattern is timed)
    pflatg = torch.zeros(play.padded_numel, dtype=torch.float32, device=dev).normal_(0, 1e-3)
    ppk = torch.zeros(play.packed_numel, dtype=torch.float32, device=dev)
    play4 = fcdp.fcdp_layout_build(pcfg.numel, pcfg.trainable, pcfg.G, 4)
    play4.prepare()
    fg_ptrs = fcdp.pointer_array([pflatg] * pcfg.G)
    torch.cuda.synchronize()

    def unfused():
        for _ in range(pcfg.G):
            fcdp.fcdp_pack_trainable(play4, pflatg, ppk, compute)
        fcdp.fcdp_reduce_grad_shard(pg_ptrs, pcfg.G, 0, pS, fcdp.F32, fcdp.F32, pshard, compute)

    # whole-model layout: the LoRA parameters of all layers packed in one launch
    wl = pcfg.layers
    wlay = fcdp.fcdp_layout_build(list(pcfg.numel) * wl, list(pcfg.trainable) * wl, pcfg.G, 2)
    wlay.prepare()
    wflat = torch.zeros(wlay.padded_numel, dtype=torch.bfloat16, device=dev).normal_(0, 0.02)
    wpacked = torch.zeros(wlay.packed_numel, dtype=torch.bfloat16, device=dev)
    torch.cuda.synchronize()
    wpack_us = 1e3 * time_kernel(lambda: fcdp.fcdp_pack_trainable(wlay, wflat, wpacked, compute), reps=30)
    wunpack_us = 1e3 * time_kernel(lambda: fcdp.fcdp_unpack_trainable(wlay, wpacked, wflat, compute), reps=30)
    w_bytes = wlay.trainable_numel * 2
    del wflat
    unfused_us = 1e3 * time_kernel(unfused, reps=30)
    fused_us = 1e3 * time_kernel(lambda: fcdp.fcdp_reduce_trainable_shard(
        play4, fg_ptrs, 0, fcdp.F32, fcdp.F32, pshard, compute), reps=50)

    # ---- launch-bound leg: GPT-2-small layers, eager against a HIP graph --
    small = None
    if not args.no_small_leg:
        scfg = synth.CONFIGS["gpt2_small_g4"]
        slay = fcdp.fcdp_layout_build(scfg.numel, None, scfg.G, 2)
        slay.prepare()
        sL, sS, sN = 12, slay.shard_numel, slay.numel     # GPT-2-small has 12 such layers
        sflat = [torch.zeros(slay.padded_numel, dtype=torch.bfloat16, device=dev).normal_(0, 0.02)
                 for _ in range(sL)]
        ssh = [fcdp.pointer_array([f.data_ptr() + r * sS * 2 for r in range(scfg.G)]) for f in sflat]
        sten = [torch.empty((k + 7) // 8 * 8, dtype=torch.bfloat16, device=dev) for k in scfg.numel]
        sten_p = fcdp.pointer_array(sten)
        sgr = torch.zeros(scfg.G, sS, dtype=torch.float32, device=dev).normal_(0, 1e-3)
        sgr_p = fcdp.pointer_array([sgr.data_ptr() + r * sS * 4 for r in range(scfg.G)])
        sout = torch.empty(sS, dtype=torch.float32, device=dev)

        def sweep():        # backward-like sweep from resident shards: K1 + K3 per layer
            for l in range(sL - 1, -1, -1):
                fcdp.fcdp_materialize_layer(slay, fcdp.SRC_DEVICE_SHARDS, ssh[l], None, None,
                                            sten_p, False, compute, None)
                fcdp.fcdp_reduce_grad_shard(sgr_p, scfg.G, 0, sS, fcdp.F32, fcdp.F32, sout, compute)

        torch.cuda.synchronize()
        fcdp.fcdp_timing_enable(4 * sL + 8)
        sweep(); sweep()
        torch.cuda.synchronize()
        n1, t1 = fcdp.fcdp_timing_collect(fcdp.KERNEL_UNFLATTEN)
        n3, t3 = fcdp.fcdp_timing_collect(fcdp.KERNEL_REDUCE)
        fcdp.fcdp_timing_enable(0)
        eager_ms = time_kernel(sweep, reps=20)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=compute, capture_error_mode="thread_local"):
            sweep()
        with torch.cuda.stream(compute):
            graph_ms = time_kernel(graph.replay, reps=20)
        if not args.no_check:
            off = slay.offsets
            for t, k in enumerate(scfg.numel):
                assert torch.equal(sten[t][:k], sflat[0][off[t]:off[t] + k]), "graph replay mismatch"
        small = {"workload": "%s: %d layers of %.1f MB, unflatten + fp32 reduce of %d partials per layer"
                             % (scfg.name, sL, sN * 2 / 1e6, scfg.G),
                 "unflatten_kernel_us": round(1e3 * t1 / max(n1, 1), 2),
                 "reduce_kernel_us": round(1e3 * t3 / max(n3, 1), 2),
                 "eager_us_per_layer": round(1e3 * eager_ms / sL, 2),
                 "graph_us_per_layer": round(1e3 * graph_ms / sL, 2)}
        del graph, sflat, sten, sgr, sout

    # ---- CPU oracle on a bounded sample of the same workload -------------
    cpu = cpu_par = cpu_peft = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.lib()
        n_s = max(1, min(args.cpu_sample_layers, L))
        t_cpu = 0.0
        for l in range(n_s):
            flat = gathered[l].cpu().view(torch.int16).numpy().view(np.uint16)
            shards = [flat[r * S:(r + 1) * S] for r in range(G)]
            parts = [partials[l][r].cpu().numpy() for r in range(G)]
            t0 = time.perf_counter()
            tens = oracle.materialize_from_shards(shards, cfg.numel)     # forward
            H = oracle.cache_store(shards)                               # "H[p] <- p"
            tens2 = oracle.materialize_from_flat(H, cfg.numel)           # backward
            red = oracle.reduce(parts, 0, S, oracle.F32)
            t_cpu += time.perf_counter() - t0
            if l == 0 and not args.no_check:
                assert np.array_equal(tens[0], kept_tensors.get(0, tensors)[0][:cfg.numel[0]].cpu().view(torch.int16).numpy().view(np.uint16))
                assert np.array_equal(red.view(np.uint32), grad_shard.cpu().numpy().view(np.uint32))
            del tens, tens2, H, red
        # the same oracle, one layer per thread (ctypes releases the GIL): what the
        # host's cores give together, still nothing tuned
        from concurrent.futures import ThreadPoolExecutor
        n_t = max(1, min(args.cpu_threads, L, os.cpu_count() or 1))
        work = []
        for l in range(n_t):
            flat = gathered[l].cpu().view(torch.int16).numpy().view(np.uint16)
            work.append(([flat[r * S:(r + 1) * S] for r in range(G)],
                         [partials[l][r].cpu().numpy() for r in range(G)]))

        def one_layer(w):
            shards, parts = w
            H = oracle.cache_store(shards)
            return (len(oracle.materialize_from_shards(shards, cfg.numel)),
                    len(oracle.materialize_from_flat(H, cfg.numel)),
                    oracle.reduce(parts, 0, S, oracle.F32).size)

        with ThreadPoolExecutor(n_t) as pool:
            t0 = time.perf_counter()
            list(pool.map(one_layer, work))
            t_par = time.perf_counter() - t0
        del work
        # the PEFT steps of one LoRA layer on the same oracle (one thread)
        pflat_h = pflat.cpu().view(torch.int16).numpy().view(np.uint16)
        t0 = time.perf_counter()
        ppk_h = oracle.pack(pflat_h, pcfg.numel, pcfg.trainable, pcfg.G)
        t_pack = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.unpack(ppk_h, pflat_h, pcfg.numel, pcfg.trainable)
        t_unpack = time.perf_counter() - t0
        pparts = [pgrads[r].cpu().numpy() for r in range(pcfg.G)]
        t0 = time.perf_counter()
        oracle.reduce(pparts, 0, pS, oracle.F32)
        t_pred = time.perf_counter() - t0
        cpu_peft = {"pack_us": round(t_pack * 1e6, 1), "unpack_us": round(t_unpack * 1e6, 1),
                    "reduce_packed_us": round(t_pred * 1e6, 1), "cores": 1, "kind": "oracle"}
        del pflat_h, ppk_h, pparts
        cpu_par = {"value": round(2 * n_t * layer_bytes / t_par / 1e9, 3), "unit": "GB/s",
                   "cores": n_t, "kind": "oracle, one layer per thread",
                   "sample": "%d layers at once, %.1f s wall" % (n_t, t_par)}
        cpu = {"value": round(2 * n_s * layer_bytes / t_cpu / 1e9, 3), "unit": "GB/s",
               "cores": 1, "kind": "oracle",
               "sample": "%d of %d layers of %s (materialize from shards, cache store, "
                         "materialize from cache, fp32 reduce), %.1f s of CPU time, host has %d cores"
                         % (n_s, L, cfg.name, t_cpu, os.cpu_count())}

    out = {
        "metric": "layer materialize GB/s (% HBM & host-link peak); grad-shard reduce GB/s",
        "value": round(value, 3), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "dtype_note": "the only arithmetic on the path is the fp32 rank-order sum; "
        "bf16 parameters are moved as bit patterns", "data": "synthetic",
        "config": {"workload": "%s: %d layers of %d tensors, %.1f M parameters each, G=%d shards/layer, "
                               "forward unflatten + D2H cache store (%s), backward host fetch (%s) + "
                               "unflatten + fp32 reduce of %d partials"
                               % (cfg.name, L, T, N / 1e6, G, args.store, args.fetch, G),
                   "layer_bytes": layer_bytes, "fetch": args.fetch, "store": args.store},
        "roofline": {"kernel": "copy_pieces<1,3> (unflatten: forward from the gathered shards, "
                               "backward from the DMA staging buffer)", "bound": "hbm",
                     "achieved": round(k1_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(k1_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": MEASURED_TRAFFIC.get(cfg.name),
                     "bytes_per_launch": k1_bytes, "avg_launch_ms": round(k1_ms, 4),
                     "launches_timed": k1_launches},
        "roofline_reduce": {"kernel": "reduce_ranks (fp32 in, fp32 out)", "bound": "hbm",
                            "achieved": round(k3_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                            "frac": round(k3_gbps / HBM_PEAK_GBPS, 4),
                            "traffic": MEASURED_TRAFFIC_REDUCE.get(cfg.name),
                            "bytes_per_launch": k3_bytes, "avg_launch_ms": round(k3_ms, 4),
                            "launches_timed": k3_launches,
                            "bf16_out_gbps": round((G * S * 4 + S * 2) / (k3b_ms * 1e-3) / 1e9, 1),
                            "bf16_in_bf16_out_gbps": round((G * S * 2 + S * 2) / (k3bb_ms * 1e-3) / 1e9, 1)},
        "host_link": {"peak": LINK_PEAK_GBPS, "unit": "GB/s",
                      "forward_store_d2h": round(d2h_gbps, 2), "backward_fetch_h2d": round(h2d_gbps, 2),
                      "frac_d2h": round(d2h_gbps / LINK_PEAK_GBPS, 4), "frac_h2d": round(h2d_gbps / LINK_PEAK_GBPS, 4),
                      "probe_h2d": round(link["h2d"], 2), "probe_d2h": round(link["d2h"], 2),
                      # backward sweep per layer against the longer of its two parts
                      "backward_overlap_efficiency": round(
                          max(layer_bytes / (link["h2d"] * 1e9) * 1e3, k1_ms + k3_ms) / (bwd_ms / L), 4)
                      if link_fetched else None,
                      "one_layer_dma_fetch_plus_unflatten_ms": round(dma_ms, 3),
                      "one_layer_zero_copy_ms": round(zc_ms, 3),
                      "one_layer_scatter_dma_ms": round(sc_ms, 3),
                      "zero_copy_gbps": round(N * 2 / (zc_ms * 1e-3) / 1e9, 2)},
        "plain_copy_gbps": round(4 * N / (copy_ms * 1e-3) / 1e9, 1),
        "adaptive": {"tau": args.tau, "kept_layers": len(kept_sets),
                     "stored_bytes_per_step": link_stored // args.steps,
                     "fetched_bytes_per_step": link_fetched // args.steps},
        "peft": {"workload": "llama7b_lora_g8 (LoRA r16 on q,v): per layer", "pack_us": round(pack_us, 2),
                 "unpack_us": round(unpack_us, 2), "reduce_packed_us": round(pred_us, 2),
                 "grad_shard_from_flat_grads_us": {"G_packs_then_reduce": round(unfused_us, 2),
                                                   "fused_reduce_trainable_shard": round(fused_us, 2)},
                 "trainable_bytes": play.trainable_numel * 2, "cpu_oracle": cpu_peft,
                 "whole_model_%d_layers" % wl: {"trainable_bytes": w_bytes, "pack_us": round(wpack_us, 2),
                                                "unpack_us": round(wunpack_us, 2),
                                                "pack_gbps": round(2 * w_bytes / (wpack_us * 1e-6) / 1e9, 1)}},
        "small_layers": small,
        "cpu_baseline": cpu,
        "cpu_baseline_all_threads": cpu_par,
    }
    cache.free()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
