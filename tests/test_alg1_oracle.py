"""Pins for the Alg. 1 replay oracle against what the paper states in prose
(Sec. 4.3, Sec. 4.5) and its traffic model (Sec. 6.2, Sec. 6.3)."""
import os

from oracle import alg1

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _records(key):
    out = []
    with open(os.path.join(GOLDEN, "paper_closed_forms.txt")) as f:
        for line in f:
            w = line.split()
            if w and w[0] == key:
                out.append(w)
    return out


def _stack(L, frozen_numel, trainable_numel):
    return [[("base", frozen_numel, False), ("lora", trainable_numel, True)]
            if frozen_numel else [("w", trainable_numel, True)]
            for _ in range(L)]


def test_full_finetune_traffic_is_2W():
    """Sec. 6.2: forward W + backward 0 + reduce-scatter W = 2W per iteration
    (ZeRO-3: 3W), every iteration, since all parameters are dirty again after
    each step."""
    rec = _records("traffic_full")[0]
    L, n = 6, 1000
    tr = alg1.replay(_stack(L, 0, n), iterations=4)
    W = L * n
    for v in tr["inter_elems"]:
        assert v == {"fwd": W, "bwd": 0, "rs": W}
        assert (v["fwd"] + v["bwd"] + v["rs"]) / W == float(rec[4])
    zero3 = W + W + W            # gather twice, reduce-scatter once (Sec. 2.1)
    assert zero3 / W == float(rec[2])
    assert tr["stale_reads"] == 0


def test_peft_traffic_is_2Wt_after_first_iteration():
    """Sec. 4.5 / Sec. 6.3: iteration 1 gathers everything once; from
    iteration 2 only trainable parameters take the inter-node path."""
    rec = _records("traffic_peft")[0]
    frac = float(rec[2])
    L, Wl = 8, 100000
    wt = int(Wl * frac)
    tr = alg1.replay(_stack(L, Wl - wt, wt), iterations=5)
    W, Wt = L * Wl, L * wt
    assert tr["inter_elems"][0] == {"fwd": W, "bwd": 0, "rs": Wt}
    for v in tr["inter_elems"][1:]:
        assert v == {"fwd": Wt, "bwd": 0, "rs": Wt}
    zero3_peft = 2 * W + Wt
    fcdp_comm = 2 * Wt
    assert abs(zero3_peft / fcdp_comm - float(rec[4])) / float(rec[4]) < 0.01
    assert tr["stale_reads"] == 0


def test_sources_per_phase():
    """Which source serves each parameter (Alg. 1's two branches)."""
    tr = alg1.replay(_stack(3, 50, 5), iterations=3)
    ev = tr["events"]
    # iteration 1: everything misses in forward, is stored, hits in backward
    for l in range(3):
        for name in ("base", "lora"):
            assert (0, "fwd", l, name, alg1.INTER) in ev
            assert (0, "fwd", l, name, "store") in ev
            assert (0, "bwd", l, name, alg1.HOST) in ev
    # later: frozen hits in forward, trainable misses; backward always hits
    for it in (1, 2):
        for l in range(3):
            assert (it, "fwd", l, "base", alg1.HOST) in ev
            assert (it, "fwd", l, "base", alg1.INTER) not in ev
            assert (it, "fwd", l, "lora", alg1.INTER) in ev
            assert (it, "bwd", l, "lora", alg1.HOST) in ev
            assert (it, "bwd", l, "base", alg1.HOST) in ev
    # backward never uses the inter-node gather (Sec. 4.3)
    assert not [e for e in ev if e[1] == "bwd" and e[4] == alg1.INTER]
    # backward visits layers L..1
    bw = [e[2] for e in ev if e[0] == 0 and e[1] == "bwd" and e[3] == "base"]
    assert bw == [2, 1, 0]
    # at the end only trainable parameters are dirty
    assert all(d == (k[1] == "lora") for k, d in tr["dirty"].items())


def test_adaptive_placement_limits():
    """Sec. 4.4: tau near 0 forces every layer to host memory (the plain
    schedule: one store and one load per layer), tau near 100 % keeps
    everything on the device (no PCIe traffic); in between, fewer bytes move
    the higher tau is."""
    sizes = [100, 200, 300, 400, 500]
    W = sum(sizes)

    def util(it, l):                 # activations pile up through the forward pass
        return 0.30 + 0.12 * l

    low = alg1.replay_adaptive(sizes, util, 0.0, 2)["iterations"]
    assert all(r == {"kept": [], "stored": W, "fetched": W} for r in low)
    high = alg1.replay_adaptive(sizes, util, 1.0, 2)["iterations"]
    assert all(r == {"kept": [0, 1, 2, 3, 4], "stored": 0, "fetched": 0} for r in high)
    mid = alg1.replay_adaptive(sizes, util, 0.55, 1)["iterations"][0]
    assert mid["kept"] == [0, 1, 2] and mid["stored"] == 900 and mid["fetched"] == 900
    moved = [alg1.replay_adaptive(sizes, util, t / 20, 1)["iterations"][0]["stored"] for t in range(21)]
    assert moved == sorted(moved, reverse=True) and moved[0] == W and moved[-1] == 0
