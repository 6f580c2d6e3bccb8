"""Discrete-event model of one synchronisation round of data-parallel training
through a parameter server (Sec. 3 and Sec. 4.2 of the P3 paper), used to put
a measured update cost next to a network in the paper's pipeline picture and
to look at the slice-size trade-off of Sec. 5.7.  CPU only; no GPU code is
involved and nothing here is on the library's hot path.

The picture (Sec. 3): backward propagation runs from the last layer to the
first and releases layer l's gradients when its backward step ends.  A unit of
synchronisation (a whole layer, or a slice of at most `slice_elems` parameters,
Sec. 4.2) then passes three stages, each of which handles one unit at a time
and never interrupts it: gradient propagation (push, the uplink), parameter
update (the server) and parameter propagation (pull, the downlink).  The next
forward step of layer l starts when the forward step of layer l-1 has ended and
every unit of layer l has come back.

A stage picks its next unit among those waiting for it either in arrival order
(first come, first served: the baseline of Sec. 3) or most urgent first
(priority = position of the parent layer in forward order, slices of a layer in
ascending offset: Sec. 4, Sec. 4.2).  Three policies:

    "layer_fifo"   whole layers, arrival order        (baseline)
    "slice_fifo"   slices, arrival order              (slicing only, Sec. 5.3)
    "p3"           slices, most urgent first          (P3)

Stage times are linear in the unit's size: fixed + elems * per_elem, given per
stage as (fixed_seconds, seconds_per_element).
"""
from __future__ import annotations

import argparse
import heapq
import json
from dataclasses import dataclass, field

POLICIES = ("layer_fifo", "slice_fifo", "p3")
STAGES = ("push", "update", "pull")


@dataclass
class Unit:
    uid: int            # position in (layer, offset) order = urgency, smaller first
    layer: int
    elems: int
    ready: float        # when the gradients exist
    start: list = field(default_factory=lambda: [0.0, 0.0, 0.0])
    end: list = field(default_factory=lambda: [0.0, 0.0, 0.0])


def make_units(layers, slice_elems, sliced):
    """Units in (layer, offset) order.  Slicing rule of Sec. 4.2: full slices of
    slice_elems and one shorter remainder; a layer not larger than the threshold
    is one unit."""
    units = []
    for l, n in enumerate(layers):
        n = int(n)
        if not sliced or n <= slice_elems:
            units.append(Unit(len(units), l, n, 0.0))
            continue
        off = 0
        while off < n:
            units.append(Unit(len(units), l, min(slice_elems, n - off), 0.0))
            off += slice_elems
    return units


def simulate(layers, backward, forward, stage_cost, policy="p3", slice_elems=50000):
    """One backward pass, the synchronisation of all layers, and the forward pass
    of the next iteration.

    layers      parameter counts in forward order
    backward    seconds of each layer's backward step (executed L-1 .. 0 from t=0)
    forward     seconds of each layer's forward step
    stage_cost  {"push": (fixed, per_elem), "update": (...), "pull": (...)}
    Returns a dict: units (with per-stage start/end), layer_back (when layer l is
    fully pulled), forward_start/forward_end per layer, backward_end,
    delay (start of the next forward pass minus end of backward), makespan
    (end of the next forward pass), busy (per stage: total service time).
    """
    if policy not in POLICIES:
        raise ValueError(f"unknown policy {policy!r}")
    L = len(layers)
    if not (len(backward) == L and len(forward) == L):
        raise ValueError("backward and forward need one entry per layer")
    units = make_units(layers, slice_elems, sliced=policy != "layer_fifo")
    urgent_first = policy == "p3"

    t = 0.0
    ready_at = [0.0] * L
    for l in range(L - 1, -1, -1):
        t += float(backward[l])
        ready_at[l] = t
    backward_end = t
    for u in units:
        u.ready = ready_at[u.layer]

    cost = [(float(stage_cost[s][0]), float(stage_cost[s][1])) for s in STAGES]

    def service(stage, u):
        return cost[stage][0] + cost[stage][1] * u.elems

    # event queue: (time, sequence, kind, stage, unit id); kind 0 = gradients of a unit exist, 1 = a stage finishes
    ev, seq = [], 0
    for u in units:
        heapq.heappush(ev, (u.ready, seq, 0, 0, u.uid))
        seq += 1
    waiting = [[], [], []]          # per stage: heap of (key, uid); key = arrival sequence, or urgency
    free = [True, True, True]
    arrivals = [0, 0, 0]
    busy = [0.0, 0.0, 0.0]

    def arrive(stage, uid):
        key = uid if urgent_first else arrivals[stage]
        arrivals[stage] += 1
        heapq.heappush(waiting[stage], (key, uid))

    while ev:
        now = ev[0][0]
        # everything that happens at this instant happens before any stage chooses, so that units
        # which become available together compete with each other
        while ev and ev[0][0] == now:
            _, _, kind, stage, uid = heapq.heappop(ev)
            if kind == 0:
                arrive(0, uid)
            else:
                free[stage] = True
                if stage < 2:
                    arrive(stage + 1, uid)
        for stage in range(3):
            if free[stage] and waiting[stage]:
                _, uid = heapq.heappop(waiting[stage])
                u = units[uid]
                u.start[stage] = now
                u.end[stage] = now + service(stage, u)
                busy[stage] += u.end[stage] - now
                free[stage] = False
                heapq.heappush(ev, (u.end[stage], seq, 1, stage, uid))     # a zero-time stage ends in a later
                seq += 1                                                   # round of this same instant

    layer_back = [0.0] * L
    for u in units:
        layer_back[u.layer] = max(layer_back[u.layer], u.end[2])
    forward_start, forward_end = [0.0] * L, [0.0] * L
    prev = backward_end
    for l in range(L):
        forward_start[l] = max(prev, layer_back[l])
        forward_end[l] = forward_start[l] + float(forward[l])
        prev = forward_end[l]
    return {
        "policy": policy, "units": units, "layer_back": layer_back, "backward_end": backward_end,
        "forward_start": forward_start, "forward_end": forward_end,
        "delay": forward_start[0] - backward_end, "makespan": forward_end[-1],
        "busy": dict(zip(STAGES, busy)),
    }


# ------------------------------------------------------------------ set-ups ----
def link_cost(gbps, bytes_per_elem=4, per_message_us=0.0):
    """(fixed, per_elem) of a network stage: a link of `gbps` gigabit per second
    carrying bytes_per_elem per parameter, plus a fixed cost per message."""
    return (per_message_us * 1e-6, bytes_per_elem * 8.0 / (gbps * 1e9))


MI355X_DRAIN_TBPS = 6.69      # VGG-19, W=8 fp32: 6.896 GB in 1.031 ms (kernel time; see profiles/)


def hbm_update_cost(W=8, grad_bytes=4, hbm_TBps=MI355X_DRAIN_TBPS, per_slice_ns=9.0):
    """(fixed, per_elem) of the update stage when it is the drain kernel of this
    library: W*grad_bytes + 16 bytes of HBM traffic per parameter at the rate
    `hbm_TBps` (pass the rate measured for the workload; the default is the one of
    VGG-19, W=8 fp32 on MI355X), and the selector's time per slice."""
    return (per_slice_ns * 1e-9, (W * grad_bytes + 16) / (hbm_TBps * 1e12))


def split_compute(layers, total_seconds, how="uniform"):
    """Per-layer compute times that add up to total_seconds: the same for every
    layer, or in proportion to the parameter count."""
    L = len(layers)
    if how == "uniform":
        return [total_seconds / L] * L
    if how == "by_params":
        n = float(sum(layers))
        return [total_seconds * x / n for x in layers]
    raise ValueError(how)


def sweep(layers, backward, forward, stage_cost, slice_sizes):
    """makespan and delay of the three policies over slice sizes (layer_fifo does not depend on them)."""
    rows = []
    base = simulate(layers, backward, forward, stage_cost, "layer_fifo")
    for S in slice_sizes:
        row = {"slice_elems": S, "layer_fifo": (base["makespan"], base["delay"])}
        for pol in ("slice_fifo", "p3"):
            r = simulate(layers, backward, forward, stage_cost, pol, S)
            row[pol] = (r["makespan"], r["delay"])
        rows.append(row)
    return rows


def main(argv=None):
    from . import synthetic as sy
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--workload", default="vgg19", choices=sorted(sy.CONFIGS))
    ap.add_argument("--gbps", type=float, default=10.0, help="network bandwidth per direction")
    ap.add_argument("--per-message-us", type=float, default=1.0, help="fixed cost of one push or pull message")
    ap.add_argument("--compute-ms", type=float, default=100.0, help="backward time of one iteration (forward: half)")
    ap.add_argument("--compute-split", default="uniform", choices=("uniform", "by_params"))
    ap.add_argument("--update", default="mi355x", choices=("mi355x", "link"),
                    help="update stage: this library's measured drain rate, or as slow as the link (a CPU server)")
    ap.add_argument("--drain-TBps", type=float, default=MI355X_DRAIN_TBPS,
                    help="HBM rate of the drain kernel for --update mi355x (measured: bench.py, roofline.achieved)")
    ap.add_argument("--slice-elems", type=int, nargs="*", default=[1000, 10000, 50000, 500000, 5000000])
    a = ap.parse_args(argv)
    cfg = sy.config(a.workload)
    layers = cfg["layers"]
    link = link_cost(a.gbps, 4, a.per_message_us)
    upd = (hbm_update_cost(cfg["W"], 2 if cfg["dtype"] == "bf16" else 4, a.drain_TBps) if a.update == "mi355x"
           else link)
    cost = {"push": link, "update": upd, "pull": link}
    bwd = split_compute(layers, a.compute_ms * 1e-3, a.compute_split)
    fwd = split_compute(layers, a.compute_ms * 0.5e-3, a.compute_split)
    out = {"workload": a.workload, "gbps": a.gbps, "per_message_us": a.per_message_us, "compute_ms": a.compute_ms,
           "update": a.update,
           "rows": [{"slice_elems": r["slice_elems"],
                     **{p: {"iteration_ms": round(r[p][0] * 1e3, 3), "delay_ms": round(r[p][1] * 1e3, 3)}
                        for p in POLICIES}} for r in sweep(layers, bwd, fwd, cost, a.slice_elems)]}
    print(json.dumps(out, indent=1))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
