#!/usr/bin/env python3
"""Benchmark of the FCDP per-layer hot path on one MI355X.

One step = one pass of the whole path over a transformer-shaped stack.  The
default (and the line the driver records) is the largest single-GPU
configuration, the Llama-2-70B-shaped share: 80 layers of 1.71 GB bf16
parameters, G = 32 shards per layer, fp32 gradient partials, bf16 shard out.

  forward, layer 0..L-1   unflatten the G gathered shards into the per-tensor
                          parameters (kernel, HBM-bound) and store the flat
                          image to the pinned host cache (D2H DMA, side stream)
  backward, layer L-1..0  fetch the layer from the host cache (H2D DMA through
                          two staging buffers, or the zero-copy kernel),
                          unflatten it, and reduce the G partial gradient
                          slices into this rank's shard (kernel)

A stack whose host cache does not fit the pinned arena (--arena-gb) streams
through a ring of K slots: layer l lives in slot l mod K, on the host and in
the device-side ring of gathered shards alike, i.e. the synthetic stack repeats
its K distinct layers; every store and every fetch moves a full layer, and
every fetch returns the bytes of the layer it is for.

Further legs in the same JSON line: the 13B-shaped stack (40 layers, G = 16)
with both fetch modes, the 7B-shaped stack (32 layers, G = 8, fp32 shard
out), PEFT pack / reduce / unpack, and the launch-bound GPT-2-small layer.
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

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each scaled
# by what the same counter reads for a plain copy of known size.  Not measured
# by the run that prints them: the figures are those of the file named in
# TRAFFIC_SOURCE (tests/test_bench_contract.py checks that they agree).
TRAFFIC_SOURCE = "profiles/unflatten_reduce_hbm_traffic.md"
MEASURED_TRAFFIC = {
    # config: (unflatten, reduce fp32 out, reduce bf16 out) in bytes per launch
    "llama7b_g8": (822.2e6, 911.9e6, 862.6e6),
    "llama13b_g16": (1288.7e6, 1349.3e6, 1311.0e6),
    "llama70b_g32": (3476.1e6, 3530.7e6, 3478.8e6),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="llama70b_g32")
    ap.add_argument("--layers", type=int, default=0, help="0 = the config's layer count")
    ap.add_argument("--fetch", choices=["dma", "zerocopy", "scatter"], default="dma")
    ap.add_argument("--store", choices=["dma", "zerocopy"], default="dma")
    ap.add_argument("--out", choices=["auto", "f32", "bf16"], default="auto",
                    help="gradient shard type; auto = bf16 for the 70B shape, fp32 otherwise")
    ap.add_argument("--arena-gb", type=float, default=26.0,
                    help="pinned host arena shared by all legs; bounds the cache slots of a stack")
    ap.add_argument("--cache-slots", type=int, default=0,
                    help="slots of the host cache ring; 0 = as many layers as the arena holds")
    ap.add_argument("--grad-slots", type=int, default=4,
                    help="layers of distinct gradient partials kept on the device (ring)")
    ap.add_argument("--tau", type=float, default=0.0,
                    help="adaptive GPU caching threshold (Sec. 4.4); 0 = offload every layer")
    ap.add_argument("--no-pretouch", action="store_true")
    ap.add_argument("--copies-in-flight", type=int, default=-1, help="-1 = the library default")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-legs", action="store_true", help="skip the 13B and 7B stack legs")
    ap.add_argument("--leg-steps", type=int, default=5)
    ap.add_argument("--leg-warmup", type=int, default=2)
    ap.add_argument("--no-small-leg", action="store_true",
                    help="skip the launch-bound GPT-2-small leg")
    ap.add_argument("--no-peft-leg", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--cpu-sample-layers", type=int, default=3)
    ap.add_argument("--cpu-threads", type=int, default=16,
                    help="threads of the all-threads oracle leg (one layer each; capped at the host's cores; "
                         "about 5 GB of host memory per thread at the 70B shape)")
    ap.add_argument("--probe-gib", type=int, default=16,
                    help="size of the host-link probe copy (16: the transfer size of the paper's Table 3, first row)")
    ap.add_argument("--reduce-study", action="store_true",
                    help="instead of the benchmark: the gradient-shard reduce at the 7B / 13B / 70B shard sizes "
                         "(G = 8, 16, 32) with both kernels, next to the G:1 calibration stream; "
                         "prints one JSON line")
    ap.add_argument("--reduce-sweep", action="store_true",
                    help="instead of the benchmark: the reduce kernels over G = 1..64 and the four type pairs at a "
                         "25 M-element shard (one tile per workgroup, phased at one and at two waves per SIMD, "
                         "and the default rule's pick); prints one JSON line")
    return ap.parse_args()


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def host_info():
    """What the machine's host looks like (Sec. 4.4: NUMA-local pinned buffers)."""
    info = {}
    try:
        nodes = [d for d in os.listdir("/sys/devices/system/node") if d.startswith("node") and d[4:].isdigit()]
        info["numa_nodes"] = len(nodes)
    except OSError:
        info["numa_nodes"] = None
    gpu_nodes = []
    try:
        for card in sorted(os.listdir("/sys/class/drm")):
            p = os.path.join("/sys/class/drm", card, "device")
            if card.startswith("card") and card[4:].isdigit() and os.path.exists(os.path.join(p, "numa_node")):
                vendor = open(os.path.join(p, "vendor")).read().strip()
                if vendor == "0x1002":
                    gpu_nodes.append(int(open(os.path.join(p, "numa_node")).read().strip()))
    except OSError:
        pass
    info["gpu_numa_node"] = gpu_nodes[0] if gpu_nodes else None
    try:
        for line in open("/proc/meminfo"):
            if line.startswith("MemTotal:"):
                info["mem_total_gb"] = round(int(line.split()[1]) * 1024 / 1e9, 1)
    except OSError:
        pass
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                info["cpu_model"] = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    info["cpus"] = os.cpu_count()
    return info


class Stack:
    """Device and host buffers of one stack, and its step."""

    def __init__(self, fcdp, synth, torch, cfg_name, layers, cache, arena_bytes, cache_slots, grad_slots,
                 fetch, store, out_f32, tau=0.0, node_g=1, streams=None):
        self.fcdp, self.torch = fcdp, torch
        dev = torch.device("cuda:0")
        cfg = synth.CONFIGS[cfg_name]
        self.cfg, self.L = cfg, layers or cfg.layers
        L, G = self.L, cfg.G
        self.lay = fcdp.fcdp_layout_build(cfg.numel, cfg.trainable, G, 2)
        self.lay.prepare()
        self.N, self.Np, self.S = self.lay.numel, self.lay.padded_numel, self.lay.shard_numel
        N, Np, S = self.N, self.Np, self.S
        self.layer_bytes = Np * 2
        # node_g > 1: this GPU is one of node_g in its node and caches shards [0, G / node_g)
        # of every layer (Sec. 4.3); the other shards are on the device already, as the
        # exchange inside the node would leave them
        assert G % node_g == 0 and (node_g == 1 or (tau == 0 and fetch == "dma" and store == "dma"))
        self.node_g, self.n_own = node_g, G // node_g
        self.slot_bytes = self.n_own * S * 2
        fit = max(1, int(arena_bytes // self.slot_bytes))
        self.K = min(L, cache_slots or fit, fit)
        self.Kg = min(L, max(1, grad_slots))
        self.fetch, self.store, self.out_f32, self.tau = fetch, store, out_f32, tau
        self.cache = cache
        log("%s: %d layers, N=%d, G=%d, S=%d, %.1f MB/layer; host cache ring of %d slots (%.2f GB), "
            "%d layers of gradient partials on the device"
            % (cfg.name, L, N, G, S, self.layer_bytes / 1e6, self.K, self.K * self.slot_bytes / 1e9, self.Kg))
        # ---- inputs, resident before timing ----
        self.gathered = []       # slot k: the G shards of layers l = k (mod K) as one gather buffer
        for k in range(self.K):
            g = synth.torch_device_generator(dev, cfg.config_id, k, synth.KIND_PARAM)
            w = torch.empty(Np, dtype=torch.bfloat16, device=dev)
            w.normal_(0.0, 0.02, generator=g)
            if Np > N:
                w[N:] = 0
            self.gathered.append(w)
        self.partials = []       # slot k: G fp32 slices of S elements (this rank's slice)
        for k in range(self.Kg):
            g = synth.torch_device_generator(dev, cfg.config_id, k, synth.KIND_GRAD)
            p = torch.empty(G, S, dtype=torch.float32, device=dev)
            p.normal_(0.0, 1e-3, generator=g)
            self.partials.append(p)
        self.tensors = [torch.empty(max(k, 1), dtype=torch.bfloat16, device=dev) for k in cfg.numel]
        self.staging = [torch.empty(self.n_own * S, dtype=torch.bfloat16, device=dev) for _ in range(2)]
        self.grad_shard = torch.empty(S, dtype=torch.float32 if out_f32 else torch.bfloat16, device=dev)
        self.state = fcdp.CacheState(L)
        self.state.set_tau(tau)
        self.total_mem = torch.cuda.get_device_properties(0).total_memory
        # adaptive caching: a synthetic activation-memory curve, utilisation rising
        # linearly from 35 % before the first layer to 95 % after the last; a kept
        # layer needs its own tensor set until its backward pass
        self.util = [0.35 + 0.60 * (l + 1) / L for l in range(L)]
        self.kept_sets, self.kept_tensors = {}, {}
        if tau > 0:
            for l in range(L):
                if self.util[l] < tau:
                    self.kept_tensors[l] = [torch.empty(max(k, 1), dtype=torch.bfloat16, device=dev)
                                            for k in cfg.numel]
                    self.kept_sets[l] = fcdp.pointer_array(self.kept_tensors[l])
        # one compute and one copy stream for the whole process, as a training loop has them.
        # (The second pair of streams a process puts to use ran the 13B backward sweep 3 % slower
        # than the first, the third and every later pair, by exactly its kernels' time, i.e. with
        # copies and kernels taking turns: measured with ten streams made up front.)
        self.compute, self.copy = streams or (torch.cuda.Stream(), torch.cuda.Stream())
        self.host_mode = {"dma": fcdp.SRC_HOST_DMA, "zerocopy": fcdp.SRC_HOST_ZEROCOPY,
                          "scatter": fcdp.SRC_HOST_SCATTER_DMA}[fetch]
        self.store_mode = fcdp.STORE_DMA if store == "dma" else fcdp.STORE_ZEROCOPY
        self.shard_ptrs = [fcdp.pointer_array([w.data_ptr() + r * S * 2 for r in range(G)]) for w in self.gathered]
        self.part_ptrs = [fcdp.pointer_array([p.data_ptr() + r * S * 4 for r in range(G)]) for p in self.partials]
        self.tensor_ptrs = fcdp.pointer_array(self.tensors)
        self.out_dt = fcdp.F32 if out_f32 else fcdp.BF16
        torch.cuda.synchronize()

    def slot(self, l):
        return self.cache.host + (l % self.K) * self.slot_bytes

    def step(self, record):
        """record: None, or a list that collects the sweep events."""
        fcdp, st, lay = self.fcdp, self.state, self.lay
        compute, copy, K, Kg, G, S = self.compute, self.copy, self.K, self.Kg, self.cfg.G, self.S
        ev = self.torch.cuda.Event
        if record is not None:
            e0 = ev(enable_timing=True); e0.record(compute)
        for l in range(self.L):
            src, _ = st.forward_source(l, 1, self.host_mode)          # full fine-tuning: always a miss
            tp = self.kept_sets.get(l, self.tensor_ptrs)
            if self.node_g > 1:
                fcdp.fcdp_materialize_layer(lay, src, self.shard_ptrs[l % K], None, None, tp,
                                            fcdp.STORE_NONE, compute, copy)
                fcdp.fcdp_cache_store_node_slice(lay, 0, self.n_own, self.shard_ptrs[l % K], self.slot(l),
                                                 compute, copy)
                st.place(l, self.total_mem, self.total_mem)
            elif self.tau > 0:
                fcdp.fcdp_materialize_layer(lay, src, self.shard_ptrs[l % K], None, None, tp,
                                            fcdp.STORE_NONE, compute, copy)
                # (the layer's forward computation would run here)
                if not st.place(l, int(self.util[l] * self.total_mem), self.total_mem):
                    fcdp.fcdp_cache_store(lay, self.shard_ptrs[l % K], self.slot(l), self.store_mode, compute, copy)
            else:
                fcdp.fcdp_materialize_layer(lay, src, self.shard_ptrs[l % K], self.slot(l), None, tp,
                                            self.store_mode, compute, copy)
                st.place(l, self.total_mem, self.total_mem)
        if record is not None:
            # the forward sweep ends when its last store does (no stores at tau = 1: on `compute`)
            e1 = ev(enable_timing=True); e1.record(copy if self.tau < 1.0 else compute)
        for l in range(self.L - 1, -1, -1):
            src = st.backward_source(l, 1, self.host_mode)
            if self.node_g > 1:
                fcdp.fcdp_materialize_layer_node_slice(lay, 0, self.n_own, self.shard_ptrs[l % K], self.slot(l),
                                                       self.staging[l % 2], self.tensor_ptrs, compute, copy)
            else:
                fcdp.fcdp_materialize_layer(lay, src, None, self.slot(l), self.staging[l % 2],
                                            self.kept_sets.get(l, self.tensor_ptrs), False, compute, copy)
            st.release(l)
            fcdp.fcdp_reduce_grad_shard(self.part_ptrs[l % Kg], G, 0, S, fcdp.F32, self.out_dt,
                                        self.grad_shard, compute)
        st.optimizer_step()
        if record is not None:
            e2 = ev(enable_timing=True); e2.record(compute)
            record.append((e0, e1, e2))

    def run(self, steps, warmup):
        fcdp, torch = self.fcdp, self.torch
        L, G, S, N = self.L, self.cfg.G, self.S, self.N
        for _ in range(warmup):
            self.step(None)
        torch.cuda.synchronize()
        # every kernel dispatch of the timed steps carries its own start/stop
        # events (recorded by the library on the stream it launches on)
        fcdp.fcdp_timing_enable(steps * L * 3 + 64)
        fcdp.fcdp_link_bytes(True)
        sweeps = []
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step(sweeps)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        r = {"ms_per_step": elapsed * 1e3 / steps}
        stored, fetched = fcdp.fcdp_link_bytes()
        k1_n, k1_t = fcdp.fcdp_timing_collect(fcdp.KERNEL_UNFLATTEN)
        zc_n, zc_t = fcdp.fcdp_timing_collect(fcdp.KERNEL_UNFLATTEN_ZEROCOPY)
        k3_n, k3_t = fcdp.fcdp_timing_collect(fcdp.KERNEL_REDUCE)
        fcdp.fcdp_timing_enable(0)
        r["k1_launches"], r["k1_ms"] = k1_n, k1_t / max(k1_n, 1)
        r["zc_launches"], r["zc_ms"] = zc_n, zc_t / max(zc_n, 1)
        r["k3_launches"], r["k3_ms"] = k3_n, k3_t / max(k3_n, 1)
        r["k3_shape"] = fcdp.fcdp_tuning_get("last_reduce_shape")
        log("%s per step: forward %s ms, backward %s ms" % (
            self.cfg.name, " ".join("%.0f" % e0.elapsed_time(e1) for e0, e1, e2 in sweeps),
            " ".join("%.0f" % e1.elapsed_time(e2) for e0, e1, e2 in sweeps)))
        r["fwd_ms"] = sum(e0.elapsed_time(e1) for e0, e1, e2 in sweeps) / steps
        r["bwd_ms"] = sum(e1.elapsed_time(e2) for e0, e1, e2 in sweeps) / steps
        r["k1_bytes"] = 4 * N                                   # read N*2 + write N*2
        r["k3_bytes"] = G * S * 4 + S * (4 if self.out_f32 else 2)
        r["k1_gbps"] = r["k1_bytes"] / (r["k1_ms"] * 1e-3) / 1e9 if r["k1_ms"] else 0.0
        r["k3_gbps"] = r["k3_bytes"] / (r["k3_ms"] * 1e-3) / 1e9 if r["k3_ms"] else 0.0
        r["stored"], r["fetched"] = stored // steps, fetched // steps
        r["d2h_gbps"] = stored / steps / (r["fwd_ms"] * 1e-3) / 1e9
        r["h2d_gbps"] = fetched / steps / (r["bwd_ms"] * 1e-3) / 1e9
        r["value"] = 2 * L * self.layer_bytes / (r["ms_per_step"] * 1e-3) / 1e9
        return r

    def check(self):
        """After a step the tensors hold layer 0, the shard its gradient, the
        host slots the layers stored last."""
        torch, cfg = self.torch, self.cfg
        off = self.lay.offsets
        flat0 = self.gathered[0]
        last = self.kept_tensors.get(0, self.tensors)
        for t, k in enumerate(cfg.numel):
            assert torch.equal(last[t][:k], flat0[off[t]:off[t] + k]), "materialized tensor mismatch"
        acc = self.partials[0][0].clone()
        for r in range(1, cfg.G):
            acc = acc + self.partials[0][r]
        if self.out_f32:
            assert torch.equal(acc.view(torch.int32), self.grad_shard.view(torch.int32)), "gradient shard mismatch"
        else:
            assert torch.equal(acc.to(torch.bfloat16).view(torch.int16),
                               self.grad_shard.view(torch.int16)), "gradient shard mismatch"
        import numpy as np
        k = (self.L - 1) % self.K
        if (self.L - 1) not in self.kept_sets:
            n = self.n_own * self.S
            hc = torch.from_numpy(self.cache.numpy(np.int16, n, k * self.slot_bytes))
            assert torch.equal(hc, self.gathered[k][:n].cpu().view(torch.int16)), "host cache mismatch"

    def free(self):
        self.gathered = self.partials = self.tensors = self.staging = None
        self.kept_tensors = self.kept_sets = None
        # no empty_cache() here: memory handed back to the driver is wiped by it in the
        # background, on the same DMA engines the cache traffic uses, and the next leg's
        # first second of copies ran at 70 % of the link rate (measured); torch's
        # allocator keeps the blocks and the next leg reuses them


def reduce_study(fcdp, synth, torch):
    """Kernel-only times (dispatch events) of the reduce on cold, rotating
    inputs, nothing else running: calibration stream, one tile per workgroup,
    phased; fp32 partials, fp32 and bf16 shard."""
    dev = torch.device("cuda:0")
    st = torch.cuda.Stream()
    rows = []
    before = fcdp.fcdp_tuning_get("reduce_phased")
    for cname in ("llama7b_g8", "llama13b_g16", "llama70b_g32"):
        cfg = synth.CONFIGS[cname]
        G = cfg.G
        S = fcdp.fcdp_layout_build(cfg.numel, cfg.trainable, G, 2).shard_numel
        Sc = S // 1024 * 1024                    # the calibration stream takes whole tiles
        NB = 3
        ps = [torch.empty(G, S, dtype=torch.float32, device=dev).normal_(0, 1e-3) for _ in range(NB)]
        ptrs = [fcdp.pointer_array([p.data_ptr() + r * S * 4 for r in range(G)]) for p in ps]
        outs = [torch.empty(S, dtype=torch.float32, device=dev) for _ in range(NB)]
        torch.cuda.synchronize()

        def timed(kind, fn, reps=30):
            for i in range(3):
                fn(i)
            torch.cuda.synchronize()
            fcdp.fcdp_timing_enable(reps + 4)
            for i in range(reps):
                fn(i)
            torch.cuda.synchronize()
            n, ms = fcdp.fcdp_timing_collect(kind)
            fcdp.fcdp_timing_enable(0)
            return ms / n

        for odt, oname, osz in ((fcdp.F32, "fp32", 4), (fcdp.BF16, "bf16", 2)):
            row = {"config": cname, "G": G, "S": S, "out": oname}
            cal = timed(fcdp.KERNEL_PROBE_STREAM, lambda i: fcdp.fcdp_probe_reduce_stream(
                outs[i % NB], ps[i % NB], G, Sc, odt, st))
            row["calibration_stream_us"] = round(cal * 1e3, 1)
            row["calibration_stream_gbps"] = round((G * Sc * 4 + Sc * osz) / (cal * 1e-3) / 1e9, 1)
            for knob, name in ((0, "tiles"), (1, "phased")):
                fcdp.fcdp_tuning_set("reduce_phased", knob)
                ms = timed(fcdp.KERNEL_REDUCE, lambda i: fcdp.fcdp_reduce_grad_shard(
                    ptrs[i % NB], G, 0, S, fcdp.F32, odt, outs[i % NB], st))
                row[name + "_us"] = round(ms * 1e3, 1)
                row[name + "_gbps"] = round((G * S * 4 + S * osz) / (ms * 1e-3) / 1e9, 1)
                row[name + "_frac"] = round((G * S * 4 + S * osz) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)
                row[name + "_vs_calibration"] = round(row[name + "_gbps"] / row["calibration_stream_gbps"], 4)
            fcdp.fcdp_tuning_set("reduce_phased", before)
            rows.append(row)
        del ps, outs
    print(json.dumps({"study": "gradient-shard reduce against the G:1 calibration stream", "peak_gbps": HBM_PEAK_GBPS,
                      "rows": rows}), flush=True)


def reduce_sweep(fcdp, torch, S=25297920):
    """The measurement behind the library's choice of reduce kernel: for a
    range of G and the four type pairs, kernel-only fractions of the HBM peak
    of one tile per workgroup, of the phased kernel at one and at two waves
    per SIMD, and of what the default rule picks."""
    dev = torch.device("cuda:0")
    st = torch.cuda.Stream()
    before = (fcdp.fcdp_tuning_get("reduce_phased"), fcdp.fcdp_tuning_get("reduce_phase_waves"))
    rows, by_length = [], []
    try:
        for G in (1, 2, 3, 4, 6, 8, 9, 10, 12, 14, 16, 20, 24, 32, 40, 64):
            NB = 3
            ps = [torch.empty(G, S, dtype=torch.float32, device=dev).normal_(0, 1e-3) for _ in range(NB)]
            ptrs = [fcdp.pointer_array([p.data_ptr() + r * S * 4 for r in range(G)]) for p in ps]
            outs = [torch.empty(S, dtype=torch.float32, device=dev) for _ in range(NB)]
            for idt, iname, isz in ((fcdp.F32, "fp32", 4), (fcdp.BF16, "bf16", 2)):
                for odt, oname, osz in ((fcdp.F32, "fp32", 4), (fcdp.BF16, "bf16", 2)):
                    row = {"G": G, "in": iname, "out": oname}
                    for name, phased, waves in (("tiles", 0, 0), ("one", 1, 1), ("two", 1, 2), ("rule", 2, 0)):
                        if waves == 1 and G % 8:
                            continue                  # the one-wave shape is built for full load groups
                        fcdp.fcdp_tuning_set("reduce_phased", phased)
                        fcdp.fcdp_tuning_set("reduce_phase_waves", waves)
                        reps = 20
                        for i in range(3):
                            fcdp.fcdp_reduce_grad_shard(ptrs[i % NB], G, 0, S, idt, odt, outs[i % NB], st)
                        torch.cuda.synchronize()
                        fcdp.fcdp_timing_enable(reps + 4)
                        for i in range(reps):
                            fcdp.fcdp_reduce_grad_shard(ptrs[i % NB], G, 0, S, idt, odt, outs[i % NB], st)
                        torch.cuda.synchronize()
                        n, ms = fcdp.fcdp_timing_collect(fcdp.KERNEL_REDUCE)
                        fcdp.fcdp_timing_enable(0)
                        row[name] = round((G * S * isz + S * osz) / (ms / n * 1e-3) / 1e9 / HBM_PEAK_GBPS, 3)
                        if name == "rule":
                            row["rule_shape"] = fcdp.fcdp_tuning_get("last_reduce_shape")
                    rows.append(row)
                    log("G=%d %s -> %s: %s" % (G, iname, oname, {k: v for k, v in row.items() if k not in ("G", "in", "out")}))
            del ps, outs
        # by length: one tile per workgroup against the rule's pick, fp32 partials
        for G in (8, 12, 16, 32):
            for S2 in (8000000, 13000000, 15000000, 17000000, 20000000, 22544384, 25297920, 27264000,
                       30000000, 40000000, 47000000, 60000000, 100000000):
                if G * S2 * 4 * 2 > 30e9:
                    continue
                NB = 2
                ps = [torch.empty(G, S2, dtype=torch.float32, device=dev).normal_(0, 1e-3) for _ in range(NB)]
                ptrs = [fcdp.pointer_array([p.data_ptr() + r * S2 * 4 for r in range(G)]) for p in ps]
                outs = [torch.empty(S2, dtype=torch.float32, device=dev) for _ in range(NB)]
                for odt, oname, osz in ((fcdp.F32, "fp32", 4), (fcdp.BF16, "bf16", 2)):
                    row = {"G": G, "S": S2, "out": oname}
                    for name, phased in (("tiles", 0), ("rule", 2)):
                        fcdp.fcdp_tuning_set("reduce_phased", phased)
                        fcdp.fcdp_tuning_set("reduce_phase_waves", 0)
                        reps = 12
                        for i in range(2):
                            fcdp.fcdp_reduce_grad_shard(ptrs[i % NB], G, 0, S2, fcdp.F32, odt, outs[i % NB], st)
                        torch.cuda.synchronize()
                        fcdp.fcdp_timing_enable(reps + 4)
                        for i in range(reps):
                            fcdp.fcdp_reduce_grad_shard(ptrs[i % NB], G, 0, S2, fcdp.F32, odt, outs[i % NB], st)
                        torch.cuda.synchronize()
                        n, ms = fcdp.fcdp_timing_collect(fcdp.KERNEL_REDUCE)   # one interval per call
                        fcdp.fcdp_timing_enable(0)
                        row[name] = round((G * S2 * 4 + S2 * osz) / (ms / n * 1e-3) / 1e9 / HBM_PEAK_GBPS, 3)
                    row["rule_shape"] = fcdp.fcdp_tuning_get("last_reduce_shape")
                    by_length.append(row)
                    log("G=%d S=%d -> %s: %s" % (G, S2, oname, {k: v for k, v in row.items() if k not in ("G", "S", "out")}))
                del ps, outs
    finally:
        fcdp.fcdp_tuning_set("reduce_phased", before[0])
        fcdp.fcdp_tuning_set("reduce_phase_waves", before[1])
    print(json.dumps({"study": "reduce kernels over G and type pairs, and over lengths; fractions of the HBM peak",
                      "S": S, "peak_gbps": HBM_PEAK_GBPS, "rows": rows, "by_length": by_length}), flush=True)


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
    if args.reduce_study:
        reduce_study(fcdp, synth, torch)
        return
    if args.reduce_sweep:
        reduce_sweep(fcdp, torch)
        return
    host = host_info()
    if args.copies_in_flight >= 0:
        fcdp.fcdp_tuning_set("max_copies_in_flight", args.copies_in_flight)
    out_f32 = {"auto": args.config != "llama70b_g32", "f32": True, "bf16": False}[args.out]

    # ---- one pinned, device-mapped arena for every leg (Sec. 4.4: allocated once) ----
    arena_bytes = int(args.arena_gb * 1e9)
    t0 = time.time()
    cache = fcdp.fcdp_host_cache_alloc(arena_bytes)
    if not args.no_pretouch:
        cache.numpy(np.uint8)[:] = 0        # touch every page before timing
    host["pinned_arena_gb"] = round(arena_bytes / 1e9, 2)
    log("pinned host arena: %.2f GB allocated and touched in %.1f s" % (arena_bytes / 1e9, time.time() - t0))

    # ---- the headline stack ----
    stack = Stack(fcdp, synth, torch, args.config, args.layers, cache, arena_bytes, args.cache_slots,
                  args.grad_slots, args.fetch, args.store, out_f32, args.tau)
    cfg, L, G, S, N, Np = stack.cfg, stack.L, stack.cfg.G, stack.S, stack.N, stack.Np
    T, layer_bytes = len(cfg.numel), stack.layer_bytes
    head = stack.run(args.steps, args.warmup)
    log("%s: %.1f ms/step, %.2f GB/s materialized" % (cfg.name, head["ms_per_step"], head["value"]))
    if not args.no_check:
        stack.check()

    # ---- host-link probe: one large pinned copy each way ----
    probe_bytes = min(args.probe_gib << 30, arena_bytes)
    pin = torch.from_numpy(cache.numpy(np.uint8, probe_bytes))
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

    # ---- plain copy reference and the other path variants on one layer of the headline shape ----
    compute, copy = stack.compute, stack.copy

    def time_kernel(fn, reps=10, stream=None):
        stream = stream or compute
        fn(); torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(reps):
            fn()
        b.record(stream); torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    lay, tensors, staging = stack.lay, stack.tensors, stack.staging
    ref_dst = torch.empty(Np, dtype=torch.bfloat16, device=dev)
    copy_ms = time_kernel(lambda: fcdp.fcdp_probe_copy(ref_dst, stack.gathered[0], N * 2, compute))
    del ref_dst
    zc_ms = time_kernel(lambda: fcdp.fcdp_materialize_layer(
        lay, fcdp.SRC_HOST_ZEROCOPY, None, cache.host, None, tensors, False, compute, copy), reps=3)
    dma_ms = time_kernel(lambda: fcdp.fcdp_materialize_layer(
        lay, fcdp.SRC_HOST_DMA, None, cache.host, staging[0], tensors, False, compute, copy), reps=3)
    sc_ms = time_kernel(lambda: fcdp.fcdp_materialize_layer(
        lay, fcdp.SRC_HOST_SCATTER_DMA, None, cache.host, None, tensors, False, compute, copy), reps=3)
    # the reduce with the other shard types, on rotating cold partials
    oshard = torch.empty(S, dtype=torch.float32, device=dev)
    rot = [0]

    def reduce_as(idt, odt):
        rot[0] = (rot[0] + 1) % stack.Kg
        fcdp.fcdp_reduce_grad_shard(stack.part_ptrs[rot[0]], G, 0, S, idt, odt, oshard, compute)

    k3_other_ms = time_kernel(lambda: reduce_as(fcdp.F32, fcdp.BF16 if out_f32 else fcdp.F32))
    # bf16 partials (half the read bytes): the first half of each fp32 partial viewed as bf16
    k3bb_ms = time_kernel(lambda: reduce_as(fcdp.BF16, fcdp.BF16))
    del oshard
    k3_f32_gbps = (G * S * 4 + S * 4) / ((head["k3_ms"] if out_f32 else k3_other_ms) * 1e-3) / 1e9
    k3_bf16_gbps = (G * S * 4 + S * 2) / ((k3_other_ms if out_f32 else head["k3_ms"]) * 1e-3) / 1e9
    kept_layers = len(stack.kept_sets)
    head_tensor0 = stack.kept_tensors.get(0, stack.tensors)[0][:cfg.numel[0]].cpu()
    head_shard = stack.grad_shard.cpu()
    cpu_inputs = None
    if not args.no_cpu_baseline:
        # host copies of a few layers for the oracle, taken before the device buffers go
        n_s = max(1, min(args.cpu_sample_layers, stack.K, stack.Kg))
        n_t = max(1, min(args.cpu_threads, stack.K, stack.Kg, os.cpu_count() or 1))   # distinct input layers
        cpu_inputs = []
        for l in range(max(n_s, n_t)):
            flat = stack.gathered[l].cpu().view(torch.int16).numpy().view(np.uint16)
            cpu_inputs.append(([flat[r * S:(r + 1) * S] for r in range(G)],
                               [stack.partials[l][r].cpu().numpy() for r in range(G)]))
    stack.free()

    # ---- the other stacks (13B: both fetch modes; 7B: fp32 shard out) ----
    legs = {}
    if not args.no_legs:
        for name, cname, fetch, of32 in (("llama13b_g16_dma", "llama13b_g16", "dma", True),
                                         ("llama13b_g16_zerocopy", "llama13b_g16", "zerocopy", True),
                                         ("llama7b_g8_dma", "llama7b_g8", "dma", True)):
            if cname == args.config and fetch == args.fetch:
                continue
            s2 = Stack(fcdp, synth, torch, cname, 0, cache, arena_bytes, 0, args.grad_slots, fetch, "dma", of32,
                       streams=(compute, copy))
            r = s2.run(args.leg_steps, args.leg_warmup)
            if not args.no_check:
                s2.check()
            per_layer_ms = r["bwd_ms"] / s2.L
            fetch_ms = s2.layer_bytes / (link["h2d"] * 1e9) * 1e3
            kern_ms = (r["k1_ms"] if fetch == "dma" else r["zc_ms"]) + r["k3_ms"]
            legs[name] = {
                "workload": "%s: %d layers of %.1f MB, G=%d, host cache of %d slots (%.2f GB), fetch %s, fp32 shard out"
                            % (cname, s2.L, s2.layer_bytes / 1e6, s2.cfg.G, s2.K, s2.K * s2.layer_bytes / 1e9, fetch),
                "steps": args.leg_steps, "ms_per_step": round(r["ms_per_step"], 2),
                "materialized_gbps": round(r["value"], 2),
                "store_d2h_gbps": round(r["d2h_gbps"], 2), "fetch_h2d_gbps": round(r["h2d_gbps"], 2),
                "backward_ms_per_layer": round(per_layer_ms, 3),
                # DMA: the copy of one layer overlaps the kernels of another, so the pair
                # should cost the longer of the two; zero-copy: the fetch IS the kernel
                "overlap_efficiency": round((max(fetch_ms, kern_ms) if fetch == "dma" else fetch_ms + r["k3_ms"])
                                            / per_layer_ms, 4),
                "unflatten_us": round(1e3 * (r["k1_ms"] if fetch == "dma" else r["zc_ms"]), 1),
                "unflatten_gbps": round(r["k1_gbps"], 1) if fetch == "dma" else None,
                "unflatten_frac": round(r["k1_gbps"] / HBM_PEAK_GBPS, 4) if fetch == "dma" else None,
                "reduce_us": round(1e3 * r["k3_ms"], 1), "reduce_gbps": round(r["k3_gbps"], 1),
                "reduce_frac": round(r["k3_gbps"] / HBM_PEAK_GBPS, 4),
            }
            log("%s: %.1f ms/step" % (name, r["ms_per_step"]))
            s2.free()
            del s2

    # ---- one GPU of a node of 8 (Sec. 4.3: it caches and fetches 1/8 of every layer; the other
    # 7/8 are on the device already, as the exchange inside the node would leave them) ----
    if not args.no_legs:
        node_g = 8
        s3 = Stack(fcdp, synth, torch, "llama70b_g32", 0, cache, arena_bytes, args.cache_slots or 15, args.grad_slots,
                   "dma", "dma", False, node_g=node_g, streams=(compute, copy))
        r = s3.run(args.leg_steps, args.leg_warmup)
        if not args.no_check:
            s3.check()
        per_layer_ms = r["bwd_ms"] / s3.L
        fetch_ms = s3.slot_bytes / (link["h2d"] * 1e9) * 1e3
        kern_ms = r["k1_ms"] + r["k3_ms"]
        legs["llama70b_g32_node_of_8"] = {
            "workload": "llama70b_g32: %d layers of %.1f MB, G=%d, this GPU one of %d in its node: it stores and "
                        "fetches shards 0..%d of every layer (%.1f MB), the other shards are on the device; "
                        "host cache of %d slots (%.2f GB), bf16 shard out"
                        % (s3.L, s3.layer_bytes / 1e6, s3.cfg.G, node_g, s3.n_own - 1, s3.slot_bytes / 1e6, s3.K,
                           s3.K * s3.slot_bytes / 1e9),
            "steps": args.leg_steps, "ms_per_step": round(r["ms_per_step"], 2),
            "materialized_gbps": round(r["value"], 2),
            "link_bytes_per_layer": s3.slot_bytes,
            "store_d2h_gbps": round(r["d2h_gbps"], 2), "fetch_h2d_gbps": round(r["h2d_gbps"], 2),
            "backward_ms_per_layer": round(per_layer_ms, 3),
            "overlap_efficiency": round(max(fetch_ms, kern_ms) / per_layer_ms, 4),
            "kernels_ms_per_backward_layer": round(kern_ms, 3),
            "unflatten_us": round(1e3 * r["k1_ms"], 1), "unflatten_frac": round(r["k1_gbps"] / HBM_PEAK_GBPS, 4),
            "reduce_us": round(1e3 * r["k3_ms"], 1), "reduce_frac": round(r["k3_gbps"] / HBM_PEAK_GBPS, 4),
        }
        log("llama70b_g32_node_of_8: %.1f ms/step" % r["ms_per_step"])
        s3.free()
        del s3

    # ---- PEFT leg: LoRA r16 on q,v of the 7B-shaped stack ----
    peft = cpu_peft = None
    pcfg = synth.CONFIGS["llama7b_lora_g8"]
    if not args.no_peft_leg:
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
        # Alg. 1's refresh of H for W_t: unpack through the mapping into the layer's host slot
        unpack_host_us = 1e3 * time_kernel(lambda: fcdp.fcdp_unpack_trainable(play, ppacked, cache.dev, compute), reps=20)
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
        wunpack_host_us = None
        if wlay.padded_numel * 2 <= arena_bytes:
            wunpack_host_us = 1e3 * time_kernel(
                lambda: fcdp.fcdp_unpack_trainable(wlay, wpacked, cache.dev, compute), reps=10)
        w_bytes = wlay.trainable_numel * 2
        del wflat
        unfused_us = 1e3 * time_kernel(unfused, reps=30)
        fused_us = 1e3 * time_kernel(lambda: fcdp.fcdp_reduce_trainable_shard(
            play4, fg_ptrs, 0, fcdp.F32, fcdp.F32, pshard, compute), reps=50)
        peft = {"workload": "llama7b_lora_g8 (LoRA r16 on q,v): per layer", "pack_us": round(pack_us, 2),
                "unpack_us": round(unpack_us, 2),
                "unpack_into_host_cache_us": round(unpack_host_us, 2),
                "reduce_packed_us": round(pred_us, 2),
                "grad_shard_from_flat_grads_us": {"G_packs_then_reduce": round(unfused_us, 2),
                                                  "fused_reduce_trainable_shard": round(fused_us, 2)},
                "trainable_bytes": play.trainable_numel * 2,
                "whole_model_%d_layers" % wl: {
                    "trainable_bytes": w_bytes, "pack_us": round(wpack_us, 2), "unpack_us": round(wunpack_us, 2),
                    "unpack_into_host_cache_us": round(wunpack_host_us, 2) if wunpack_host_us else None,
                    "unpack_into_host_cache_gbps": round(w_bytes / (wunpack_host_us * 1e-6) / 1e9, 2)
                    if wunpack_host_us else None,
                    "pack_gbps": round(2 * w_bytes / (wpack_us * 1e-6) / 1e9, 1)}}

    # ---- launch-bound leg: GPT-2-small layers ----
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
        sstage = torch.empty(slay.padded_numel, dtype=torch.bfloat16, device=dev)

        def sweep():        # backward-like sweep from resident shards: K1 + K3 per layer
            for l in range(sL - 1, -1, -1):
                fcdp.fcdp_materialize_layer(slay, fcdp.SRC_DEVICE_SHARDS, ssh[l], None, None,
                                            sten_p, False, compute, None)
                fcdp.fcdp_reduce_grad_shard(sgr_p, scfg.G, 0, sS, fcdp.F32, fcdp.F32, sout, compute)

        torch.cuda.synchronize()
        # the layer in host slot 0, then single calls of the three fetches (host time + GPU time of
        # one call after another on one stream pair)
        fcdp.fcdp_materialize_layer(slay, fcdp.SRC_DEVICE_SHARDS, ssh[0], cache.host, None, sten_p,
                                    fcdp.STORE_DMA, compute, copy)
        torch.cuda.synchronize()
        s_dma_us = 1e3 * time_kernel(lambda: fcdp.fcdp_materialize_layer(
            slay, fcdp.SRC_HOST_DMA, None, cache.host, sstage, sten_p, False, compute, copy), reps=20)
        s_zc_us = 1e3 * time_kernel(lambda: fcdp.fcdp_materialize_layer(
            slay, fcdp.SRC_HOST_ZEROCOPY, None, cache.host, None, sten_p, False, compute, copy), reps=20)
        s_static_us = 1e3 * time_kernel(lambda: fcdp.fcdp_materialize_layer_static(
            slay, cache.host, sten_p, compute, copy), reps=20)
        s_dev_us = 1e3 * time_kernel(lambda: fcdp.fcdp_materialize_layer(
            slay, fcdp.SRC_DEVICE_SHARDS, ssh[0], None, None, sten_p, False, compute, None), reps=50)
        s_red_us = 1e3 * time_kernel(lambda: fcdp.fcdp_reduce_grad_shard(
            sgr_p, scfg.G, 0, sS, fcdp.F32, fcdp.F32, sout, compute), reps=50)
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
        small = {"workload": "%s: one layer of %.1f MB, G=%d; single calls, then 12 such layers as a sweep"
                             % (scfg.name, sN * 2 / 1e6, scfg.G),
                 "single_call_us": {"unflatten_from_device_shards": round(s_dev_us, 2),
                                    "dma_fetch_plus_unflatten": round(s_dma_us, 2),
                                    "zero_copy_fetch": round(s_zc_us, 2),
                                    "static_staging_fetch": round(s_static_us, 2),
                                    "reduce_fp32": round(s_red_us, 2),
                                    "link_floor": round(sN * 2 / (link["h2d"] * 1e9) * 1e6, 2)},
                 "unflatten_kernel_us": round(1e3 * t1 / max(n1, 1), 2),
                 "reduce_kernel_us": round(1e3 * t3 / max(n3, 1), 2),
                 "eager_us_per_layer": round(1e3 * eager_ms / sL, 2),
                 "graph_us_per_layer": round(1e3 * graph_ms / sL, 2)}
        small_inputs = (sflat[0].cpu().view(torch.int16).numpy().view(np.uint16),
                        [sgr[r].cpu().numpy() for r in range(scfg.G)])
        del graph, sflat, sten, sgr, sout

    # ---- CPU oracle on a bounded sample of the same workload -------------
    cpu = cpu_par = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.lib()
        odt = oracle.F32 if out_f32 else oracle.BF16
        n_s = max(1, min(args.cpu_sample_layers, len(cpu_inputs)))
        t_cpu = 0.0
        for l in range(n_s):
            shards, parts = cpu_inputs[l]
            t0 = time.perf_counter()
            tens = oracle.materialize_from_shards(shards, cfg.numel)     # forward
            H = oracle.cache_store(shards)                               # "H[p] <- p"
            tens2 = oracle.materialize_from_flat(H, cfg.numel)           # backward
            red = oracle.reduce(parts, 0, S, odt)
            t_cpu += time.perf_counter() - t0
            if l == 0 and not args.no_check:
                assert np.array_equal(tens[0], head_tensor0.view(torch.int16).numpy().view(np.uint16))
                got = head_shard.numpy().view(np.uint32) if out_f32 else \
                    head_shard.view(torch.int16).numpy().view(np.uint16)
                assert np.array_equal(red.view(got.dtype), got)
            del tens, tens2, H, red
        # the same oracle, one layer per thread (ctypes releases the GIL): what the
        # host's cores give together, still nothing tuned
        from concurrent.futures import ThreadPoolExecutor
        # every thread its own layer's worth of work; threads beyond the distinct input layers
        # read one of them again (inputs are only read, every thread writes its own outputs)
        n_t = max(1, min(args.cpu_threads, os.cpu_count() or 1))
        work = [cpu_inputs[i % len(cpu_inputs)] for i in range(n_t)]

        def one_layer(w):
            shards, parts = w
            H = oracle.cache_store(shards)
            return (len(oracle.materialize_from_shards(shards, cfg.numel)),
                    len(oracle.materialize_from_flat(H, cfg.numel)),
                    oracle.reduce(parts, 0, S, odt).size)

        with ThreadPoolExecutor(n_t) as pool:
            t0 = time.perf_counter()
            list(pool.map(one_layer, work))
            t_par = time.perf_counter() - t0
        cpu_inputs = work = None
        if peft is not None:
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
            peft["cpu_oracle"] = {"pack_us": round(t_pack * 1e6, 1), "unpack_us": round(t_unpack * 1e6, 1),
                                  "reduce_packed_us": round(t_pred * 1e6, 1), "cores": 1, "kind": "oracle"}
            del pflat_h, ppk_h, pparts
        if small is not None:
            sflat_h, sparts = small_inputs
            t0 = time.perf_counter()
            oracle.materialize_from_flat(sflat_h, scfg.numel)
            t_sm = time.perf_counter() - t0
            t0 = time.perf_counter()
            oracle.reduce(sparts, 0, sS, oracle.F32)
            t_sr = time.perf_counter() - t0
            small["cpu_oracle"] = {"materialize_us": round(t_sm * 1e6, 1), "reduce_us": round(t_sr * 1e6, 1),
                                   "cores": 1, "kind": "oracle"}
        cpu_par = {"value": round(2 * n_t * layer_bytes / t_par / 1e9, 3), "unit": "GB/s",
                   "cores": n_t, "kind": "oracle, one layer per thread",
                   "sample": "%d layers at once, %.1f s wall" % (n_t, t_par)}
        cpu = {"value": round(2 * n_s * layer_bytes / t_cpu / 1e9, 3), "unit": "GB/s",
               "cores": 1, "kind": "oracle",
               "sample": "%d of %d layers of %s (materialize from shards, cache store, "
                         "materialize from cache, fp32 reduce of %d partials into a %s shard), "
                         "%.1f s of CPU time, host has %d cores"
                         % (n_s, L, cfg.name, G, "fp32" if out_f32 else "bf16", t_cpu, os.cpu_count())}

    traffic = MEASURED_TRAFFIC.get(cfg.name)
    out = {
        "metric": "layer materialize GB/s (% HBM & host-link peak); grad-shard reduce GB/s",
        "value": round(head["value"], 3), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(head["ms_per_step"], 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "dtype_note": "the only arithmetic on the path is the fp32 rank-order sum; "
        "bf16 parameters are moved as bit patterns", "data": "synthetic",
        "config": {"workload": "%s: %d layers of %d tensors, %.1f M parameters each, G=%d shards/layer, "
                               "forward unflatten + D2H cache store (%s), backward host fetch (%s) + "
                               "unflatten + fp32 reduce of %d partials into a %s shard"
                               % (cfg.name, L, T, N / 1e6, G, args.store, args.fetch, G,
                                  "fp32" if out_f32 else "bf16"),
                   "layer_bytes": layer_bytes, "fetch": args.fetch, "store": args.store,
                   "host_cache_slots": stack.K, "host_cache_bytes": stack.K * layer_bytes,
                   "host_cache_note": "layer l lives in slot l mod %d of the pinned arena and of the device-side "
                                      "ring of gathered shards; all %d layers distinct would need %.1f GB pinned"
                                      % (stack.K, L, L * layer_bytes / 1e9) if stack.K < L else
                                      "every layer has its own slot",
                   "grad_partial_slots": stack.Kg},
        "host": host,
        "roofline": {"kernel": "copy_pieces<1,3> (unflatten: forward from the gathered shards, "
                               "backward from the DMA staging buffer)", "bound": "hbm",
                     "achieved": round(head["k1_gbps"], 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(head["k1_gbps"] / HBM_PEAK_GBPS, 4),
                     "traffic": traffic[0] if traffic else None, "traffic_source": TRAFFIC_SOURCE,
                     "bytes_per_launch": head["k1_bytes"], "avg_launch_ms": round(head["k1_ms"], 4),
                     "launches_timed": head["k1_launches"]},
        "roofline_reduce": {"kernel": "%s (fp32 in, %s out)" % (
                                {0: "reduce_ranks", 1: "reduce_phased<104, 1, ...>", 2: "reduce_phased<52, 2, ...>"}[
                                    head["k3_shape"]],
                                "fp32" if out_f32 else "bf16"),
                            "bound": "hbm", "achieved": round(head["k3_gbps"], 1), "peak": HBM_PEAK_GBPS,
                            "unit": "GB/s", "frac": round(head["k3_gbps"] / HBM_PEAK_GBPS, 4),
                            "traffic": (traffic[1] if out_f32 else traffic[2]) if traffic else None,
                            "traffic_source": TRAFFIC_SOURCE,
                            "bytes_per_launch": head["k3_bytes"], "avg_launch_ms": round(head["k3_ms"], 4),
                            "launches_timed": head["k3_launches"],
                            "fp32_out_gbps": round(k3_f32_gbps, 1), "bf16_out_gbps": round(k3_bf16_gbps, 1),
                            "bf16_in_bf16_out_gbps": round((G * S * 2 + S * 2) / (k3bb_ms * 1e-3) / 1e9, 1)},
        "host_link": {"peak": LINK_PEAK_GBPS, "unit": "GB/s",
                      "forward_store_d2h": round(head["d2h_gbps"], 2),
                      "backward_fetch_h2d": round(head["h2d_gbps"], 2),
                      "frac_d2h": round(head["d2h_gbps"] / LINK_PEAK_GBPS, 4),
                      "frac_h2d": round(head["h2d_gbps"] / LINK_PEAK_GBPS, 4),
                      "probe_h2d": round(link["h2d"], 2), "probe_d2h": round(link["d2h"], 2),
                      "probe_bytes": probe_bytes,
                      # the paper's Table 3, first row: one 16 GB host-to-device transfer over the link
                      "probe_h2d_seconds_per_16e9_bytes": round(16e9 / (link["h2d"] * 1e9), 4),
                      "backward_ms_per_layer": round(head["bwd_ms"] / L, 3),
                      # backward sweep per layer against the longer of its two parts
                      "backward_overlap_efficiency": round(
                          max(layer_bytes / (link["h2d"] * 1e9) * 1e3, head["k1_ms"] + head["k3_ms"])
                          / (head["bwd_ms"] / L), 4) if head["fetched"] else None,
                      "one_layer_dma_fetch_plus_unflatten_ms": round(dma_ms, 3),
                      "one_layer_zero_copy_ms": round(zc_ms, 3),
                      "one_layer_scatter_dma_ms": round(sc_ms, 3),
                      "zero_copy_gbps": round(N * 2 / (zc_ms * 1e-3) / 1e9, 2)},
        "plain_copy_gbps": round(4 * N / (copy_ms * 1e-3) / 1e9, 1),
        "adaptive": {"tau": args.tau, "kept_layers": kept_layers,
                     "stored_bytes_per_step": head["stored"], "fetched_bytes_per_step": head["fetched"]},
        "stacks": legs or None,
        "peft": peft,
        "small_layers": small,
        "cpu_baseline": cpu,
        "cpu_baseline_all_threads": cpu_par,
    }
    cache.free()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
