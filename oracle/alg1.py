"""Oracle for the cache-state logic of the PEFT-aware training loop (Alg. 1).

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).

The loop is replayed step by step in the order Alg. 1 gives: initialise every
parameter dirty; forward over layers 1..L (a dirty parameter takes the
inter-node gather and refreshes the host cache H, a clean one is loaded from
H); backward over layers L..1 (always from H); one reduce-scatter of the
trainable gradients; optimizer step; trainable parameters become dirty again.
No data moves here: the replay records which source serves every parameter
and how many elements cross the node boundary, which is what Sec. 6.2 and
Sec. 6.3 count.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

INTER = "inter"   # inter-node all-gather of the rank shards (cache miss)
HOST = "host"     # host-cache load + intra-node gather (cache hit)


def replay(layers: Sequence[Sequence[Tuple[str, int, bool]]],
           iterations: int) -> Dict[str, object]:
    """layers[l] = [(param name, numel, trainable)], returns the trace.

    trace["events"]: list of (iteration, phase, layer, name, what) with phase
    in {"fwd", "bwd", "rs", "upd"}; what in {INTER, HOST, "store", "dirty"}.
    trace["inter_elems"][it] = {"fwd": e, "bwd": e, "rs": e}: elements that
    cross the node boundary in that iteration (times (N-1)/N for the exact
    per-node share, which Sec. 6.2 approximates by 1).
    """
    dirty: Dict[Tuple[int, str], bool] = {}
    H: Dict[Tuple[int, str], int] = {}      # version of the cached copy
    version: Dict[Tuple[int, str], int] = {}
    for l, layer in enumerate(layers):
        for name, _numel, _tr in layer:
            dirty[(l, name)] = True
            version[(l, name)] = 0
    events: List[tuple] = []
    vol: List[Dict[str, int]] = []
    stale_reads = 0
    for it in range(iterations):
        v = {"fwd": 0, "bwd": 0, "rs": 0}
        for l, layer in enumerate(layers):
            for name, numel, _tr in layer:
                key = (l, name)
                if dirty[key]:
                    events.append((it, "fwd", l, name, INTER))
                    v["fwd"] += numel
                    H[key] = version[key]
                    dirty[key] = False
                    events.append((it, "fwd", l, name, "store"))
                else:
                    events.append((it, "fwd", l, name, HOST))
                    if H[key] != version[key]:
                        stale_reads += 1
        for l in range(len(layers) - 1, -1, -1):
            for name, numel, _tr in layers[l]:
                key = (l, name)
                events.append((it, "bwd", l, name, HOST))
                if H[key] != version[key]:
                    stale_reads += 1
        wt = sum(numel for layer in layers for _n, numel, tr in layer if tr)
        v["rs"] = wt
        events.append((it, "rs", -1, "grad_W_t", INTER))
        for l, layer in enumerate(layers):
            for name, _numel, tr in layer:
                if tr:
                    version[(l, name)] += 1     # optimizer step changes W_t
                    dirty[(l, name)] = True
                    events.append((it, "upd", l, name, "dirty"))
        vol.append(v)
    return {"events": events, "inter_elems": vol, "stale_reads": stale_reads,
            "dirty": dict(dirty)}


def replay_adaptive(layer_bytes: Sequence[int], utilisation, tau: float,
                    iterations: int) -> Dict[str, object]:
    """Adaptive GPU caching on top of the full fine-tuning schedule (Sec. 4.4).

    layer_bytes[l]: bytes of layer l's parameters; utilisation(it, l): device
    memory utilisation in [0, 1] seen at the "cache on CPU" point of layer l,
    after its forward computation.  Below tau the layer stays on the device
    (no store, no load in the backward pass); otherwise it is stored to the
    host cache and loaded back for the backward pass.  Every parameter is
    trainable, so every forward pass starts from the gathered shards.
    Returns per-iteration kept layers and bytes over the host link.
    """
    out = []
    for it in range(iterations):
        kept, stored, fetched = [], 0, 0
        for l, nbytes in enumerate(layer_bytes):        # forward
            if utilisation(it, l) < tau:
                kept.append(l)
            else:
                stored += nbytes
        for l in range(len(layer_bytes) - 1, -1, -1):   # backward
            if l not in kept:
                fetched += layer_bytes[l]
        out.append({"kept": kept, "stored": stored, "fetched": fetched})
    return {"iterations": out}
