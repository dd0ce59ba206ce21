"""Oracle for the cache-state logic of the PEFT-aware training loop (Alg. 1).

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).

A small state machine per parameter (validity flag, parameter version, cached
version) with the three transitions the method defines -- forward use,
backward use, optimizer step -- driven through the schedule of a training
iteration (Alg. 1, Sec. 4.3, Sec. 4.5).  No data moves here: the replay
records which source serves every parameter and how many elements cross the
node boundary, which is what Sec. 6.2 and Sec. 6.3 count.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

INTER = "inter"   # inter-node all-gather of the rank shards (cache miss)
HOST = "host"     # host-cache load + intra-node gather (cache hit)


class ParamCache:
    """Cache state of one parameter: the validity flag Alg. 1 keeps for it, the
    version the optimizer has produced and the version the host copy holds.
    The three transitions are the only places the flag changes."""

    def __init__(self, numel: int, trainable: bool):
        self.numel, self.trainable = numel, trainable
        self.dirty = True          # nothing is cached before the first forward pass
        self.version = 0           # bumped by every optimizer step that touches it
        self.cached_version = None

    def forward(self) -> Tuple[str, int]:
        """Source that serves the forward pass, and elements that cross the
        node boundary for it.  A miss refreshes the host copy (Sec. 4.3,
        Sec. 4.5: trainable parameters are invalid after every step, frozen
        ones stay cached for the whole run)."""
        if self.dirty:
            self.cached_version = self.version
            self.dirty = False
            return INTER, self.numel
        return HOST, 0

    def backward(self) -> str:
        """The backward pass never leaves the node: always the host copy."""
        return HOST

    def step(self) -> bool:
        """Optimizer step: a trainable parameter changes and its cached copy
        becomes invalid; returns whether that happened."""
        if self.trainable:
            self.version += 1
            self.dirty = True
        return self.trainable

    def stale(self) -> bool:
        return self.cached_version != self.version


def replay(layers: Sequence[Sequence[Tuple[str, int, bool]]],
           iterations: int) -> Dict[str, object]:
    """layers[l] = [(param name, numel, trainable)], returns the trace.

    Drives one ParamCache per parameter through the schedule of a training
    iteration (forward over the layers in order, backward in reverse, one
    reduce-scatter of the trainable gradients, optimizer step).

    trace["events"]: list of (iteration, phase, layer, name, what) with phase
    in {"fwd", "bwd", "rs", "upd"}; what in {INTER, HOST, "store", "dirty"}.
    trace["inter_elems"][it] = {"fwd": e, "bwd": e, "rs": e}: elements that
    cross the node boundary in that iteration (times (N-1)/N for the exact
    per-node share, which Sec. 6.2 approximates by 1).
    """
    params = [[(name, ParamCache(numel, tr)) for name, numel, tr in layer] for layer in layers]
    trainable_elems = sum(pc.numel for layer in params for _n, pc in layer if pc.trainable)
    events: List[tuple] = []
    vol: List[Dict[str, int]] = []
    stale_reads = 0
    order = list(range(len(params)))
    for it in range(iterations):
        v = {"fwd": 0, "bwd": 0, "rs": 0}
        for phase, sweep in (("fwd", order), ("bwd", order[::-1])):
            for l in sweep:
                for name, pc in params[l]:
                    if phase == "fwd":
                        src, crossed = pc.forward()
                        v["fwd"] += crossed
                    else:
                        src = pc.backward()
                    events.append((it, phase, l, name, src))
                    if src == INTER:
                        events.append((it, phase, l, name, "store"))
                    elif pc.stale():
                        stale_reads += 1
        v["rs"] = trainable_elems                      # only grad W_t is reduced (Sec. 4.5, Sec. 6.3)
        events.append((it, "rs", -1, "grad_W_t", INTER))
        for l in order:
            for name, pc in params[l]:
                if pc.step():
                    events.append((it, "upd", l, name, "dirty"))
        vol.append(v)
    dirty = {(l, name): pc.dirty for l in order for name, pc in params[l]}
    return {"events": events, "inter_elems": vol, "stale_reads": stale_reads,
            "dirty": dirty}


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
