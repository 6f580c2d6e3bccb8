"""GPU parity at the full sizes of the measured workloads, in the launch
configuration bench.py times (default tile, one persistent launch per drain):
VGG-19 with 8 fp32 gradient copies, and VGG-19 with 16 bf16 copies over the
slice-size sweep under a ticked release schedule.  Every element of weights and
momentum is compared with the CPU oracle (identical bits), and the claim order
with the oracle's."""
import numpy as np
import pytest
import torch

import oracle
from oracle import OraclePlan
from paper_1905_03960_amd import binding as b
from paper_1905_03960_amd import synthetic as sy

from p3_case import DeviceCase, PAD_W, assert_same_bits, to_device

pytestmark = pytest.mark.gpu


def test_vgg19_fp32_w8_full_size_ten_iterations():
    """The configuration the bandwidth target is quoted on, for the ten iterations it names: momentum
    accumulated over ten updates of all 143,667,240 parameters, every bit against the oracle."""
    cfg = sy.config("vgg19")
    grads, w0, m0 = sy.make_inputs(cfg)
    case = DeviceCase(cfg["layers"], cfg["slice_elems"], grads, w0, m0)
    b.p3_set_hyper(case.plan, cfg["lr"], cfg["mu"])
    rw, rm = w0.copy(), m0.copy()
    for it in range(cfg["iters"]):
        case.iterate(many=True)
        oracle.sgd_whole(grads, rw, rm, cfg["lr"], cfg["mu"])
        if it in (0, 4):                              # also part of the way, so that a late error is not the only check
            case.sync()
            assert (case.order() == np.arange(case.K)).all()
            w, m = case.fetch()
            assert_same_bits(w, m, rw, rm, f"vgg19 fp32 W=8 after iteration {it + 1}")
    case.sync()
    assert (case.order() == np.arange(case.K)).all()
    w, m = case.fetch()
    assert_same_bits(w, m, rw, rm, "vgg19 fp32 W=8, ten iterations")
    # live mode on the same plan, marks arriving while the drain runs: same arithmetic, and the
    # order log is a permutation that replays against the epochs the selector observed
    b.p3_set_mode(case.plan, b.P3_MODE_LIVE)
    b.p3_begin_iter(case.plan)
    b.p3_drain(case.plan, case.stream.cuda_stream)
    for l in range(case.L - 1, -1, -1):
        b.p3_mark_ready(case.plan, l)
    b.p3_wait_layer(case.plan, 0, 20000)
    case.sync(20000)
    oracle.sgd_whole(grads, rw, rm, cfg["lr"], cfg["mu"])
    order = case.order()
    assert sorted(order.tolist()) == list(range(case.K))
    w, m = case.fetch()
    assert_same_bits(w, m, rw, rm, "vgg19 fp32 W=8 live")
    # a fourth iteration by eight servers' shares (slices round robin), one after another on the same arenas
    G = 8
    for j in range(G):
        p = b.p3_plan_sharded(cfg["layers"], cfg["slice_elems"], G, j)
        b.p3_bind(p, [t.data_ptr() for t in case.g], b.P3_GRAD_FP32, case.w.data_ptr(), case.m.data_ptr())
        b.p3_set_hyper(p, cfg["lr"], cfg["mu"])
        b.p3_begin_iter(p)
        b.p3_mark_ready_many(p, list(range(case.L - 1, -1, -1)))
        b.p3_drain(p, case.stream.cuda_stream)
        b.p3_sync(p, 20000)
        assert (b.p3_query_order(p) == np.arange(j, case.K, G)).all(), j
        b.p3_destroy(p)
    oracle.sgd_whole(grads, rw, rm, cfg["lr"], cfg["mu"])
    w, m = case.fetch()
    assert_same_bits(w, m, rw, rm, "vgg19 fp32 W=8, eight shares")


def test_vgg19_bf16_w16_slice_sweep_ticked():
    cfg = sy.config("vgg19_bf16")
    sizes = [int(x) for x in cfg["layers"]]
    grads, w0, m0 = sy.make_inputs(cfg)
    rw, rm = w0.copy(), m0.copy()
    oracle.sgd_whole(grads, rw, rm, cfg["lr"], cfg["mu"])       # the arithmetic does not depend on the slicing
    rw2, rm2 = rw.copy(), rm.copy()
    oracle.sgd_whole(grads, rw2, rm2, cfg["lr"], cfg["mu"])     # second iteration (the live repeat)
    probe = b.p3_plan(sizes, cfg["slice_elems"])
    offsets = [b.p3_layer_offset(probe, l) for l in range(len(sizes))]
    arena = b.p3_arena_elems(probe)
    b.p3_destroy(probe)
    g = [to_device(sy.flat_to_arena(x, sizes, offsets, arena, fill=np.uint16(0x7FC0))) for x in grads]
    w_init = to_device(sy.flat_to_arena(w0, sizes, offsets, arena, fill=PAD_W))
    m_init = to_device(sy.flat_to_arena(m0, sizes, offsets, arena, fill=PAD_W))
    w, m = torch.empty_like(w_init), torch.empty_like(m_init)
    stream = torch.cuda.Stream()
    for S in sy.BF16_SLICE_SWEEP:
        w.copy_(w_init)
        m.copy_(m_init)
        torch.cuda.synchronize()
        plan = b.p3_plan(sizes, S)
        assert [b.p3_layer_offset(plan, l) for l in range(len(sizes))] == offsets
        K = b.p3_num_slices(plan)
        b.p3_bind(plan, [t.data_ptr() for t in g], b.P3_GRAD_BF16, w.data_ptr(), m.data_ptr())
        b.p3_set_hyper(plan, cfg["lr"], cfg["mu"])
        release = sy.release_ticks(cfg["seed"], len(sizes), K)
        b.p3_set_mode(plan, b.P3_MODE_TICKED, release)
        b.p3_begin_iter(plan)
        for l in range(len(sizes) - 1, -1, -1):
            b.p3_mark_ready(plan, l)
        b.p3_drain(plan, stream.cuda_stream)
        b.p3_sync(plan, 20000)
        want, _ = OraclePlan(sizes, S).order_ticked(release)
        got = b.p3_query_order(plan)
        assert (got == want).all(), f"S={S}: claim order differs from the oracle's"
        gw = sy.arena_to_flat(w.cpu().numpy(), sizes, offsets)
        gm = sy.arena_to_flat(m.cpu().numpy(), sizes, offsets)
        assert_same_bits(gw, gm, rw, rm, f"vgg19 bf16 W=16 S={S}")
        if True:
            # the same release pattern in real time: a live drain, the host marking the layers in reverse
            # order with pauses in proportion to the release ticks (a few hundred microseconds in all)
            import time
            b.p3_set_mode(plan, b.P3_MODE_LIVE)
            b.p3_begin_iter(plan)
            b.p3_drain(plan, stream.cuda_stream)
            marks = list(range(len(sizes) - 1, -1, -1))
            span = float(release.max()) or 1.0
            t0 = time.perf_counter()
            for l in marks:
                while time.perf_counter() - t0 < 600e-6 * float(release[l]) / span:
                    pass
                b.p3_mark_ready(plan, l)
            b.p3_sync(plan, 20000)
            got, seen = b.p3_query_order(plan), b.p3_query_trace(plan)
            assert (OraclePlan(sizes, S).order_replay(marks, seen) == got).all(), f"S={S}: live order does not replay"
            gw = sy.arena_to_flat(w.cpu().numpy(), sizes, offsets)
            gm = sy.arena_to_flat(m.cpu().numpy(), sizes, offsets)
            assert_same_bits(gw, gm, rw2, rm2, f"vgg19 bf16 W=16 S={S}, live second iteration")
        b.p3_destroy(plan)


def test_arenas_beyond_32_bit_offsets_sampled():
    """Arenas of 2.2e9 elements (8.8 GB each: element offsets beyond 2^31, byte
    offsets beyond 2^33).  Inputs are a fixed function of the arena position, filled
    on the device; the oracle recomputes sampled positions one by one -- random
    ones, and the neighbourhoods of every power-of-two boundary, layer edge and
    slice edge -- after two snapshot iterations and a live one.  Untouched padding
    is checked too."""
    sizes, S, W = [1000, 2_200_000_000, 4097, 5_000_000], 50000, 2
    free, _ = torch.cuda.mem_get_info()
    if free < 45 << 30:
        pytest.skip("needs 45 GB of device memory")
    plan = b.p3_plan(sizes, S)
    L, K = len(sizes), b.p3_num_slices(plan)
    offs = [b.p3_layer_offset(plan, l) for l in range(L)]
    arena = b.p3_arena_elems(plan)
    assert arena > 1 << 31
    salts = list(range(W)) + [100, 200]
    scales = [-24] * W + [-20, -22]
    tens = [torch.empty(arena, dtype=torch.float32, device="cuda") for _ in range(W + 2)]
    for t, salt, sc in zip(tens, salts, scales):
        sy.pattern_fill_torch(t, salt, sc)
    g, w, m = tens[:W], tens[W], tens[W + 1]
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    b.p3_set_tuning(plan, 0, 0, 0, 20000)
    b.p3_bind(plan, [t.data_ptr() for t in g], b.P3_GRAD_FP32, w.data_ptr(), m.data_ptr())
    b.p3_set_hyper(plan, 0.1, 0.9)
    for _ in range(2):
        b.p3_begin_iter(plan)
        b.p3_mark_ready_many(plan, list(range(L - 1, -1, -1)))
        b.p3_drain(plan, stream.cuda_stream)
    b.p3_sync(plan, 20000)
    assert (b.p3_query_order(plan) == np.arange(K)).all()
    b.p3_set_mode(plan, b.P3_MODE_LIVE)
    b.p3_begin_iter(plan)
    b.p3_drain(plan, stream.cuda_stream)
    for l in range(L - 1, -1, -1):
        b.p3_mark_ready(plan, l)
    b.p3_sync(plan, 20000)
    got = b.p3_query_order(plan)
    assert sorted(got.tolist()) == list(range(K))
    torch.cuda.synchronize()

    # sampled positions inside layers
    rng = np.random.default_rng(20)
    inside = [rng.integers(o, o + n, size=60000) for o, n in zip(offs, sizes)]
    near = []
    for c in [1 << k for k in range(20, 32)] + [(1 << 31) + (1 << 30), 2_000_000_000]:
        near.append(np.arange(c - 70, c + 70))
    for o, n in zip(offs, sizes):
        near += [np.arange(o, o + 70), np.arange(o + n - 70, o + n)]
    lo1 = offs[1]
    for k in (1, 2, 1000, 20000, 43999):                     # slice edges of the big layer
        near.append(np.arange(lo1 + k * S - 40, lo1 + k * S + 40))
    idx = np.unique(np.concatenate(inside + near)).astype(np.int64)
    in_layer = np.zeros(idx.shape, dtype=bool)
    for o, n in zip(offs, sizes):
        in_layer |= (idx >= o) & (idx < o + n)
    idx = idx[in_layer & (idx < arena)]
    gs = [sy.pattern_values(idx, salt, sc) for salt, sc in zip(salts[:W], scales[:W])]
    rw, rm = sy.pattern_values(idx, salts[W], scales[W]), sy.pattern_values(idx, salts[W + 1], scales[W + 1])
    for _ in range(3):
        oracle.sgd_whole(gs, rw, rm, 0.1, 0.9)
    di = torch.from_numpy(idx).cuda()
    gw, gm = w[di].cpu().numpy(), m[di].cpu().numpy()
    assert_same_bits(gw, gm, rw, rm, "sampled positions of 8.8 GB arenas")
    # gradients are inputs: never written
    for t, salt, sc in zip(g, salts[:W], scales[:W]):
        assert (t[di].cpu().numpy().view(np.uint32) == sy.pattern_values(idx, salt, sc).view(np.uint32)).all()
    # padding between and behind the layers keeps its initial pattern
    pad = []
    for o, n, nxt in zip(offs, sizes, offs[1:] + [arena]):
        pad.append(np.arange(o + n, nxt))
    pad = np.concatenate(pad).astype(np.int64)
    if pad.size:
        dp = torch.from_numpy(pad).cuda()
        assert (w[dp].cpu().numpy().view(np.uint32) == sy.pattern_values(pad, salts[W], scales[W]).view(np.uint32)).all()
        assert (m[dp].cpu().numpy().view(np.uint32) == sy.pattern_values(pad, salts[W + 1], scales[W + 1]).view(np.uint32)).all()
    del plan
