"""GPU parity of the lean build of the drain kernel (p3_set_launch(plan, P3_LAUNCH_LEAN): workgroups of 256
lanes that leave room on their compute unit for other kernels' workgroups), against the same CPU oracle and
to the same bar as the default build: claim order bit-exact, weights and momentum identical bits."""
import time

import numpy as np
import pytest
import torch

import oracle
from oracle import OraclePlan
from paper_1905_03960_amd import binding as b
from paper_1905_03960_amd import synthetic as sy

from p3_case import DeviceCase, assert_same_bits, stream_beside

pytestmark = pytest.mark.gpu

# around the lean build's workgroup step (256 lanes x 4), its default tile (4096) and the default build's tile
RAGGED = [1, 3, 5, 10, 1023, 1024, 1025, 4095, 4096, 4097, 8191, 8193, 50001, 64, 63, 65, 12288, 2, 3327, 3328,
          3329, 2047, 2049, 255, 257, 16385]


def draw(seed, n, W, bf16=False):
    cfg = dict(seed=seed, W=W, dtype="bf16" if bf16 else "fp32", sigma_g=0.01, sigma_w=0.05, layers=[n])
    return sy.make_inputs(cfg)


def lean_case(*args, **kw):
    case = DeviceCase(*args, **kw)
    b.p3_set_launch(case.plan, b.P3_LAUNCH_LEAN)
    return case


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("W", [1, 2, 3, 4, 5, 8, 16, 17])
def test_lean_ragged_layers_every_worker_count(W, bf16):
    n = sum(RAGGED)
    grads, w0, m0 = draw(1100 + W, n, W, bf16)
    rw, rm = w0.copy(), m0.copy()
    for _ in range(2):
        oracle.sgd_whole(grads, rw, rm, 0.1, 0.9)
    for S in (50000, 1000 if W % 2 else 4096):
        case = lean_case(RAGGED, S, grads, w0, m0)
        for _ in range(2):
            case.iterate()
        assert (case.order() == np.arange(case.K)).all()
        w, m = case.fetch()
        assert_same_bits(w, m, rw, rm, f"lean W={W} bf16={bf16} S={S}")


@pytest.mark.parametrize("tile,wgs", [(0, 1), (1024, 1), (2048, 2), (65536, 1)])
def test_lean_tile_sizes_and_a_switch_between_the_builds(tile, wgs):
    sizes = [300000, 17, 70001]
    grads, w0, m0 = draw(1200, sum(sizes), 8)
    rw, rm = w0.copy(), m0.copy()
    for _ in range(4):
        oracle.sgd_whole(grads, rw, rm, 0.1, 0.9)
    case = DeviceCase(sizes, 50000, grads, w0, m0, tile_elems=tile, wgs_per_cu=wgs)
    for launch in (b.P3_LAUNCH_LEAN, b.P3_LAUNCH_LEAN, b.P3_LAUNCH_FUSED, b.P3_LAUNCH_LEAN):
        b.p3_set_launch(case.plan, launch)            # applied by the iteration that begins next
        case.iterate()
        assert (case.order() == np.arange(case.K)).all()
    w, m = case.fetch()
    assert_same_bits(w, m, rw, rm, f"lean tile={tile} wgs={wgs}")


def test_lean_live_drain_claims_what_the_replay_of_its_trace_claims():
    sizes = [40000, 300, 250000, 7, 120000, 64]
    grads, w0, m0 = draw(1300, sum(sizes), 4)
    case = lean_case(sizes, 4096, grads, w0, m0, watchdog_ms=4000)
    b.p3_set_mode(case.plan, b.P3_MODE_LIVE)
    o = OraclePlan(sizes, 4096)
    rw, rm = w0.copy(), m0.copy()
    for it, gap in enumerate([0.0, 0.002, 0.0]):
        marks = list(range(len(sizes) - 1, -1, -1)) if it < 2 else [3, 0, 5, 1, 4, 2]
        b.p3_begin_iter(case.plan)
        b.p3_drain(case.plan, case.stream.cuda_stream)       # the kernel starts with nothing ready
        for l in marks:
            time.sleep(gap)
            b.p3_mark_ready(case.plan, l)
        b.p3_sync(case.plan, 5000)
        got, seen = case.order(), b.p3_query_trace(case.plan)
        assert sorted(got.tolist()) == list(range(case.K))
        assert (o.order_replay(marks, seen) == got).all()    # every claim was the most urgent ready slice
        oracle.sgd_whole(grads, rw, rm, 0.1, 0.9)
    w, m = case.fetch()
    assert_same_bits(w, m, rw, rm, "lean live")


def test_lean_live_drain_shares_the_device_with_the_stream_that_produces_its_gradients():
    """No compute unit is reserved: the producer's kernels (copies that write the gradients, the marks) have to
    find room beside the resident drain workgroups.  If they did not, the drain would sit on the whole device
    until its watchdog ends it, and the sync below would report that."""
    sizes = [40000, 300, 250000, 7, 120000, 64, 600000]
    L = len(sizes)
    grads, w0, m0 = draw(1400, sum(sizes), 4)
    case = lean_case(sizes, 4096, grads, w0, m0, watchdog_ms=5000)
    b.p3_set_mode(case.plan, b.P3_MODE_LIVE)
    staged = [t.clone() for t in case.g]                      # the real gradients, kept aside
    producer = stream_beside(case.stream)
    o = OraclePlan(sizes, 4096)
    rw, rm = w0.copy(), m0.copy()
    for it in range(3):
        marks = list(range(L - 1, -1, -1)) if it != 1 else [3, 0, 6, 5, 1, 4, 2]
        for t in case.g:
            t.view(torch.int32).fill_(0x7FC00000)              # NaN until produced
        torch.cuda.synchronize()
        b.p3_begin_iter(case.plan)
        b.p3_drain(case.plan, case.stream.cuda_stream)        # resident before the first gradient exists
        with torch.cuda.stream(producer):
            torch.cuda._sleep(2_000_000)
            for l in marks:
                lo, n = case.offsets[l], case.sizes[l]
                for k in range(len(case.g)):
                    case.g[k][lo:lo + n].copy_(staged[k][lo:lo + n], non_blocking=True)
                b.p3_mark_ready_on_stream(case.plan, l, producer.cuda_stream)
        b.p3_sync(case.plan, 8000)
        got, seen = case.order(), b.p3_query_trace(case.plan)
        assert sorted(got.tolist()) == list(range(case.K))
        assert (o.order_replay(marks, seen) == got).all()
        oracle.sgd_whole(grads, rw, rm, 0.1, 0.9)
    w, m = case.fetch()
    assert_same_bits(w, m, rw, rm, "lean live beside its producer")   # a slice taken too early would be NaN


def test_lean_fifo_policy_and_ticked_mode():
    sizes = [30000, 12, 90000, 5000, 77]
    L = len(sizes)
    grads, w0, m0 = draw(1500, sum(sizes), 2)
    case = lean_case(sizes, 2048, grads, w0, m0)
    o = OraclePlan(sizes, 2048)
    rel = sy.release_ticks(1500, L, case.K)
    b.p3_set_mode(case.plan, b.P3_MODE_TICKED, rel)
    rw, rm = w0.copy(), m0.copy()
    case.iterate()
    want, _ = o.order_ticked(rel)
    assert (case.order() == want).all()
    oracle.sgd_whole(grads, rw, rm, 0.1, 0.9)
    b.p3_set_policy(case.plan, b.P3_POLICY_FIFO)
    case.iterate()
    want, _ = o.order_ticked_fifo(rel)
    assert (case.order() == want).all()
    oracle.sgd_whole(grads, rw, rm, 0.1, 0.9)
    w, m = case.fetch()
    assert_same_bits(w, m, rw, rm, "lean ticked + fifo")


def test_lean_queue_longer_than_the_run_ring_and_state_in_device_memory():
    """The lean build keeps fewer run records (256) and a smaller ready bitmap (65,536 slices) in LDS.  A
    look-ahead of one tile gives thousands of runs, several times the ring; 2,500 layers are more than the
    selector's LDS table holds, so bitmap and layer states stay in device memory."""
    sizes = [300000, 500, 250000, 40, 1000]
    grads, w0, m0 = draw(1600, sum(sizes), 2)
    case = lean_case(sizes, 256, grads, w0, m0, lookahead=1, watchdog_ms=8000)
    assert case.K > 2000
    b.p3_set_mode(case.plan, b.P3_MODE_LIVE)
    o = OraclePlan(sizes, 256)
    rw, rm = w0.copy(), m0.copy()
    for marks in ([4, 3, 2, 1, 0], [2, 0, 4, 1, 3]):
        b.p3_begin_iter(case.plan)
        b.p3_drain(case.plan, case.stream.cuda_stream)
        for l in marks:
            b.p3_mark_ready(case.plan, l)
        b.p3_sync(case.plan, 8000)
        got, seen = case.order(), b.p3_query_trace(case.plan)
        assert (o.order_replay(marks, seen) == got).all()
        oracle.sgd_whole(grads, rw, rm, 0.1, 0.9)
    w, m = case.fetch()
    assert_same_bits(w, m, rw, rm, "lean live, long queue")

    rng = np.random.default_rng(5)
    sizes, S = [int(x) for x in rng.integers(1, 400, size=2500)], 64
    grads, w0, m0 = draw(1601, sum(sizes), 2)
    case = lean_case(sizes, S, grads, w0, m0, watchdog_ms=8000)
    o = OraclePlan(sizes, S)
    L = len(sizes)
    first, second = list(range(L - 1, L // 2, -1)), list(range(L // 2, -1, -1))
    b.p3_begin_iter(case.plan)
    b.p3_mark_ready_many(case.plan, first)
    b.p3_drain(case.plan, case.stream.cuda_stream)
    b.p3_mark_ready_many(case.plan, second)
    b.p3_drain(case.plan, case.stream.cuda_stream)
    assert (case.order() == o.order_snapshot(first + [-1] + second + [-1])).all()
    rw, rm = w0.copy(), m0.copy()
    oracle.sgd_whole(grads, rw, rm, 0.1, 0.9)
    w, m = case.fetch()
    assert_same_bits(w, m, rw, rm, "lean, state in device memory")

    sizes = [50000, 7, 30001]                                  # one slice per parameter: 80,008 slices
    grads, w0, m0 = draw(1602, sum(sizes), 2)
    case = lean_case(sizes, 1, grads, w0, m0, watchdog_ms=8000)
    assert case.K > 65536
    case.iterate([1, 2, 0])
    assert (case.order() == np.arange(case.K)).all()
    rw, rm = w0.copy(), m0.copy()
    oracle.sgd_whole(grads, rw, rm, 0.1, 0.9)
    w, m = case.fetch()
    assert_same_bits(w, m, rw, rm, "lean, bitmap in device memory")


def test_lean_full_size_vgg19_iteration():
    """The parameter set the benchmark times, one snapshot iteration of the lean build at full size."""
    cfg = sy.config("vgg19")
    grads, w0, m0 = sy.make_inputs(cfg)
    case = lean_case(cfg["layers"], cfg["slice_elems"], grads, w0, m0)
    b.p3_set_hyper(case.plan, cfg["lr"], cfg["mu"])
    case.iterate(many=True)
    assert (case.order() == np.arange(case.K)).all()
    rw, rm = w0.copy(), m0.copy()
    oracle.sgd_whole(grads, rw, rm, cfg["lr"], cfg["mu"])
    w, m = case.fetch()
    assert_same_bits(w, m, rw, rm, "lean vgg19")
