"""Pins for the oracle's planner and processing order (CPU only).

Each test checks the oracle against something other than itself: the paper's
worked example, closed forms, or a brute-force scan written independently here.
"""
import os

import numpy as np
import pytest

from oracle import OraclePlan


def read_golden(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split(":", 1)
            out[k.strip()] = [float(x) if "." in x else int(x) for x in v.split()]
    return out


# ------------------------------------------------------------------ planner --
@pytest.mark.parametrize("sizes,S", [
    ([10], 3), ([1, 1, 1], 1), ([200704, 256, 65536, 256, 2560, 10], 50000),
    ([5, 50000, 50001, 99999, 100000, 100001], 50000), ([7, 3], 100),
])
def test_planner_partitions_every_layer(sizes, S):
    """Slices tile each layer exactly, none exceeds the threshold, only the
    last slice of a layer may be short, and ids ascend with (layer, offset)
    (Sec. 4.2: the threshold is the maximum slice size; Sec. 4: slices inherit
    the layer's priority)."""
    p = OraclePlan(sizes, S)
    layer, off, ln = p.slice_table()
    assert p.L == len(sizes) and p.N == sum(sizes)
    assert p.K == sum(-(-n // S) for n in sizes)        # ceil(n/S), by integer arithmetic
    assert (np.diff(layer) >= 0).all()
    for l, n in enumerate(sizes):
        sel = layer == l
        assert off[sel][0] == 0
        assert (off[sel][1:] == off[sel][:-1] + ln[sel][:-1]).all()   # contiguous
        assert off[sel][-1] + ln[sel][-1] == n                        # covers the layer
        assert (ln[sel][:-1] == S).all() and 1 <= ln[sel][-1] <= S


def test_planner_slice_counts_of_paper_models():
    """Slice counts at the paper's slice size of 50,000 (Sec. 5.7) for the
    paper's models, from ceil(n/S) summed by hand-checkable arithmetic."""
    from paper_1905_03960_amd import synthetic as sy
    vgg = sy.vgg19_layers()
    assert sum(vgg) == 143667240 and len(vgg) == 38
    assert abs(max(vgg) / sum(vgg) - 0.715) < 5e-4          # Sec. 3: 71.5 % in one FC layer
    assert OraclePlan(vgg, 50000).K == 2902
    rn = sy.resnet50_layers()
    assert sum(rn) == 25557032 and len(rn) == 161
    assert OraclePlan(rn, 50000).K == 643
    s2s = sy.seq2seq_layers()
    assert sum(s2s) == 58367232 and len(s2s) == 15 and s2s[0] == max(s2s)
    assert OraclePlan(s2s, 50000).K == 1175
    assert [OraclePlan(vgg, S).K for S in sy.BF16_SLICE_SWEEP] == [35091, 2902, 317, 65]


def test_planner_rejects_bad_arguments():
    for sizes, S in [([], 4), ([0], 4), ([3, -1], 4), ([3], 0)]:
        with pytest.raises(ValueError):
            OraclePlan(sizes, S)


# ------------------------------------------------------------- closed forms --
SHAPES = [([200704, 256, 65536, 256, 2560, 10], 50000), ([9, 1, 30, 4, 17], 4), ([3] * 40, 1)]


@pytest.mark.parametrize("sizes,S", SHAPES)
def test_all_marked_then_one_drain_is_identity(sizes, S):
    p = OraclePlan(sizes, S)
    ev = list(range(p.L - 1, -1, -1)) + [-1]
    assert (p.order_snapshot(ev) == np.arange(p.K)).all()


@pytest.mark.parametrize("sizes,S", SHAPES)
def test_drain_after_each_mark_gives_reverse_layers(sizes, S):
    p = OraclePlan(sizes, S)
    layer, _, _ = p.slice_table()
    ev = []
    for l in range(p.L - 1, -1, -1):
        ev += [l, -1]
    got = p.order_snapshot(ev)
    want = np.concatenate([np.nonzero(layer == l)[0] for l in range(p.L - 1, -1, -1)])
    assert (got == want).all()


def test_drain_with_nothing_ready_claims_nothing():
    p = OraclePlan([5, 5], 2)
    assert p.order_snapshot([-1]).size == 0
    assert (p.order_snapshot([-1, 1, -1, -1, 0, -1]) == [3, 4, 5, 0, 1, 2]).all()


def test_snapshot_rejects_double_mark_and_bad_layer():
    p = OraclePlan([5, 5], 2)
    with pytest.raises(ValueError):
        p.order_snapshot([0, 0, -1])
    with pytest.raises(ValueError):
        p.order_snapshot([2, -1])


# --------------------------------------------------- the paper's own example --
def test_three_layer_example_of_the_paper(golden_dir):
    g = read_golden(os.path.join(golden_dir, "three_layer_example.txt"))
    p = OraclePlan(g["layer_sizes"], g["slice_elems"][0])
    layer, _, _ = p.slice_table()
    end_bwd = g["backward_end_tick"][0]

    order, tick = p.order_ticked(g["release_ticks"])
    assert list(order) == g["p3_order"]
    done = [int(tick[layer[order] == l].max()) + 1 for l in range(p.L)]
    assert done == g["p3_layer_complete"]
    assert done[0] - end_bwd == g["p3_delay_units"][0]
    # every layer is back no later than the next forward pass reaches it
    assert all(d <= need for d, need in zip(done, g["p3_layer_needed_by"]))

    forder, ftick = p.order_ticked_fifo(g["release_ticks"])
    assert list(forder) == g["fifo_order"]
    fdone = [int(ftick[layer[forder] == l].max()) + 1 for l in range(p.L)]
    assert fdone == g["fifo_layer_complete"]
    assert fdone[0] - end_bwd == g["fifo_delay_units"][0]
    # the paper's two statements: delay = 2 x sync time of first layer; halved by priorities
    assert g["fifo_delay_units"][0] == 2 * g["sync_units_per_layer"][0]
    assert 2 * g["p3_delay_units"][0] == g["fifo_delay_units"][0]


# ------------------------------------------------ brute force: minimum ready --
def brute_force_ticked(sizes, S, release):
    """Independent restatement with Python sets: at each step the claimed slice
    must be the minimum of (released and not yet claimed)."""
    ids = []
    g = 0
    for l, n in enumerate(sizes):
        k = -(-n // S)
        ids.append(list(range(g, g + k)))
        g += k
    pending = {l: release[l] for l in range(len(sizes)) if release[l] >= 0}
    avail, clock, out = set(), 0, []
    while pending or avail:
        for l in [l for l, r in pending.items() if r <= clock]:
            avail.update(ids[l])
            del pending[l]
        if not avail:
            clock = min(pending.values())
            continue
        pick = min(avail)
        avail.remove(pick)
        out.append(pick)
        clock += 1
    return out


@pytest.mark.parametrize("seed", range(12))
def test_ticked_order_equals_brute_force(seed):
    rng = np.random.default_rng(seed)
    L = int(rng.integers(1, 9))
    sizes = [int(x) for x in rng.integers(1, 40, size=L)]
    S = int(rng.integers(1, 12))
    release = [int(x) for x in rng.integers(0, 30, size=L)]
    if seed % 3 == 0 and L > 1:
        release[int(rng.integers(0, L))] = -1            # a layer that is never released
    p = OraclePlan(sizes, S)
    order, tick = p.order_ticked(release)
    assert list(order) == brute_force_ticked(sizes, S, release)
    assert (np.diff(tick) >= 1).all()
    released_slices = sum(-(-n // S) for n, r in zip(sizes, release) if r >= 0)
    assert len(order) == released_slices == len(set(order.tolist()))


def test_ticked_preemption_and_non_preemption():
    """A more urgent layer released later overtakes the REMAINING slices of a
    less urgent one (Sec. 1.1) but never the slice already taken (Sec. 4.2)."""
    p = OraclePlan([3, 6], 1)                 # layer 0: ids 0..2, layer 1: ids 3..8
    order, _ = p.order_ticked([2, 0])
    assert list(order) == [3, 4, 0, 1, 2, 5, 6, 7, 8]


def test_ticked_idle_jump():
    p = OraclePlan([2, 2], 1)
    order, tick = p.order_ticked([10, 0])
    assert list(order) == [2, 3, 0, 1] and list(tick) == [0, 1, 10, 11]


def test_priority_is_nondecreasing_between_readiness_changes():
    """Between two consecutive releases the claimed layer index never decreases."""
    rng = np.random.default_rng(99)
    sizes = [int(x) for x in rng.integers(1, 200, size=20)]
    p = OraclePlan(sizes, 7)
    layer, _, _ = p.slice_table()
    release = np.sort(rng.integers(0, p.K, size=p.L))[::-1].copy()
    order, tick = p.order_ticked(release)
    assert sorted(order.tolist()) == list(range(p.K))            # a permutation
    edges = sorted(set(int(r) for r in release))
    for lo, hi in zip(edges, edges[1:] + [10 ** 9]):
        seg = layer[order[(tick >= lo) & (tick < hi)]]
        assert (np.diff(seg) >= 0).all()


# --------------------------------------------------------------------- replay --
def test_replay_reproduces_snapshot_and_ticked_orders():
    p = OraclePlan([9, 1, 30, 4, 17], 4)
    layer, _, _ = p.slice_table()
    marks = [4, 3, 2, 1, 0]
    # all marks seen before the first claim -> identity
    assert (p.order_replay(marks, [5] * p.K) == np.arange(p.K)).all()
    # one more mark seen at every claim, as in a drain-per-mark run
    ev = []
    for l in marks:
        ev += [l, -1]
    want = p.order_snapshot(ev)
    seen = [marks.index(int(layer[g])) + 1 for g in want]
    assert (p.order_replay(marks, seen) == want).all()


def test_replay_rejects_impossible_traces():
    p = OraclePlan([2, 2], 1)
    with pytest.raises(ValueError):
        p.order_replay([1, 0], [0])            # nothing ready at the first claim
    with pytest.raises(ValueError):
        p.order_replay([1, 0], [2, 1])         # observed marks cannot decrease
    with pytest.raises(ValueError):
        p.order_replay([1, 0], [1, 1, 1])      # layer 1 has only two slices


def test_fifo_comparison_policy_ties_follow_backward_order():
    p = OraclePlan([2, 2], 1)
    order, _ = p.order_ticked_fifo([0, 0])
    assert list(order) == [2, 3, 0, 1]


# ------------- first come, first served: release order other than backward order --
def test_fifo_hand_worked_cases(golden_dir):
    """Non-monotone release ticks, an idle server in between, and a backlog in which a layer
    released later (but before the server is free) waits its turn: Sec. 3's aggressive
    synchronisation, layers whole in the order backward hands them over."""
    g = read_golden(os.path.join(golden_dir, "fifo_hand_cases.txt"))
    p = OraclePlan(g["layer_sizes"], g["slice_elems"][0])
    for case in "ab":
        order, tick = p.order_ticked_fifo(g[f"{case}_release_ticks"])
        assert list(order) == g[f"{case}_fifo_order"], case
        assert list(tick) == g[f"{case}_claim_ticks"], case
    p = OraclePlan(g["c_layer_sizes"], g["slice_elems"][0])
    order, tick = p.order_ticked_fifo(g["c_release_ticks"])
    assert list(order) == g["c_fifo_order"] and list(tick) == g["c_claim_ticks"]


def brute_force_fifo(sizes, S, release):
    """Independent restatement as a tick-by-tick simulation of a waiting line: at every tick the
    layers released at that tick join the line (later layer first among them, as backward
    produces them); the server, when free, takes the head of the line and is busy one tick per
    slice.  Returns (slice ids in service order, tick at which each was served)."""
    ids, g = [], 0
    for n in sizes:
        k = -(-n // S)
        ids.append(list(range(g, g + k)))
        g += k
    line, out, ticks = [], [], []
    todo = sum(1 for r in release if r >= 0)
    in_service = []                                   # slices of the layer being served, not yet served
    t = 0
    while todo or line or in_service:
        for l in sorted((l for l, r in enumerate(release) if r == t), reverse=True):
            line.append(l)
            todo -= 1
        if not in_service and line:
            in_service = list(ids[line.pop(0)])
        if in_service:
            out.append(in_service.pop(0))
            ticks.append(t)
        t += 1
    return out, ticks


@pytest.mark.parametrize("seed", range(12))
def test_fifo_order_equals_brute_force(seed):
    rng = np.random.default_rng(1000 + seed)
    L = int(rng.integers(1, 9))
    sizes = [int(x) for x in rng.integers(1, 40, size=L)]
    S = int(rng.integers(1, 12))
    # spans longer than the work (idle gaps), shorter (backlog), and equal ticks
    release = [int(x) for x in rng.integers(0, [4, 30, 120][seed % 3], size=L)]
    if seed % 4 == 0 and L > 1:
        release[int(rng.integers(0, L))] = -1            # a layer that is never released
    p = OraclePlan(sizes, S)
    order, tick = p.order_ticked_fifo(release)
    want, want_ticks = brute_force_fifo(sizes, S, release)
    assert list(order) == want and list(tick) == want_ticks
