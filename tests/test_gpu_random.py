"""GPU parity over seeded random combinations of what the other tests vary one at a time: layer lists, slice
size, number and type of gradient copies, launch kind (two launches, one persistent launch, the lean build),
tile size, workgroups per compute unit, weight decay, mode (snapshot in one or two drains, live, ticked) and
policy.  Two iterations each; claim order bit-exact against the oracle, weights and momentum identical bits."""
import time

import numpy as np
import pytest

import oracle
from oracle import OraclePlan
from paper_1905_03960_amd import binding as b
from paper_1905_03960_amd import synthetic as sy

from p3_case import DeviceCase, assert_same_bits

pytestmark = pytest.mark.gpu


def arrival_order(o, marks):
    """Layers whole, in mark order: the oracle's first-come-first-served order with release = arrival rank."""
    release = np.zeros(o.L, dtype=np.int64)
    for rank, l in enumerate(marks):
        release[l] = rank
    return o.order_ticked_fifo(release)[0]


def one_case(seed):
    rng = np.random.default_rng(seed)
    L = int(rng.integers(1, 14))
    sizes = [int(min(400000, max(1, round(10 ** rng.uniform(0, 5.6))))) for _ in range(L)]
    small = sum(sizes) < 60000                       # one-parameter slices only where that stays a few thousand slices
    S = int(rng.choice([1, 3, 64, 1000, 4096, 50000, 1 << 20] if small else [1000, 4096, 50000, 1 << 20]))
    W = int(rng.choice([1, 2, 3, 4, 5, 8, 16, 17]))
    bf16 = bool(rng.integers(0, 2))
    launch = int(rng.integers(0, 3))
    mode = str(rng.choice(["snapshot", "two drains", "live", "ticked"]))
    policy = int(rng.integers(0, 2))
    tile = int(rng.choice([0, 0, 1024, 2048, 8192]))
    wgs = int(rng.choice([0, 1, 2]))
    wd = float(rng.choice([0.0, 0.0, 1e-2]))
    what = (f"seed {seed}: L={L} N={sum(sizes)} S={S} W={W} bf16={bf16} launch={launch} mode={mode} "
            f"policy={policy} tile={tile} wgs={wgs} wd={wd}")
    cfg = dict(seed=5000 + seed, W=W, dtype="bf16" if bf16 else "fp32", sigma_g=0.01, sigma_w=0.05,
               layers=[sum(sizes)])
    grads, w0, m0 = sy.make_inputs(cfg)
    case = DeviceCase(sizes, S, grads, w0, m0, tile_elems=tile, wgs_per_cu=wgs, watchdog_ms=4000)
    b.p3_set_launch(case.plan, launch)
    b.p3_set_hyper(case.plan, 0.1, 0.9, 1.0, wd)
    b.p3_set_policy(case.plan, policy)
    o = OraclePlan(sizes, S)
    rw, rm = w0.copy(), m0.copy()
    for it in range(2):
        marks = [int(x) for x in rng.permutation(L)]
        if mode == "ticked":
            release = sy.release_ticks(seed + it, L, case.K)
            rng.shuffle(release)
            b.p3_set_mode(case.plan, b.P3_MODE_TICKED, release)
            case.iterate(marks)
            want = (o.order_ticked_fifo(release) if policy else o.order_ticked(release))[0]
            got = case.order()
        elif mode == "live":
            b.p3_set_mode(case.plan, b.P3_MODE_LIVE)
            b.p3_begin_iter(case.plan)
            b.p3_drain(case.plan, case.stream.cuda_stream)
            for l in marks:
                if rng.integers(0, 3) == 0:
                    time.sleep(0.0005)
                b.p3_mark_ready(case.plan, l)
            b.p3_sync(case.plan, 6000)
            got, seen = case.order(), b.p3_query_trace(case.plan)
            want = arrival_order(o, marks) if policy else o.order_replay(marks, seen)
        else:
            b.p3_set_mode(case.plan, b.P3_MODE_SNAPSHOT)
            cut = int(rng.integers(0, L + 1)) if mode == "two drains" else L
            b.p3_begin_iter(case.plan)
            events = []
            for part in (marks[:cut], marks[cut:]):
                if part:
                    b.p3_mark_ready_many(case.plan, part)
                    b.p3_drain(case.plan, case.stream.cuda_stream)
                    events += part + [-1]
            got = case.order()
            # first come, first served: each drain serves its own marks whole in mark order, so the two
            # drains together serve all marks in mark order
            want = arrival_order(o, marks) if policy else o.order_snapshot(events)
        assert got.shape == want.shape and (got == want).all(), f"claim order differs, {what}, iteration {it}"
        oracle.sgd_whole(grads, rw, rm, 0.1, 0.9, 1.0, wd)
    w, m = case.fetch()
    assert_same_bits(w, m, rw, rm, what)


@pytest.mark.parametrize("block", range(6))
def test_random_combinations(block):
    for seed in range(7000 + 50 * block, 7000 + 50 * (block + 1)):
        one_case(seed)
