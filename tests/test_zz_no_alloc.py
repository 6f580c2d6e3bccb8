"""The allocation-free iteration (p3_drain_static) against the bound-plan path
(p3_bind + p3_begin_iter + p3_mark_ready_many + p3_drain), both through the C
ABI, on the same seeded inputs: claim order and every weight and momentum bit
must be equal.  Two calls in a row share the GPU's static control array; the
second is smaller than the first (stale contents of the first must not leak)."""
import numpy as np
import pytest
import torch

from oracle import OraclePlan
from paper_1905_03960_amd import binding as b
from paper_1905_03960_amd import synthetic as sy

from p3_case import DeviceCase, PAD_W, assert_same_bits, to_device

pytestmark = pytest.mark.gpu


def run_static(sizes, S, grads, w0, m0, marks, lr, mu, rescale, wd, stream):
    """One call of the allocation-free entry point on fresh device copies of the inputs."""
    plan = b.p3_plan(sizes, S)                       # host only: never bound
    L, K = len(sizes), b.p3_num_slices(plan)
    offs = [b.p3_layer_offset(plan, l) for l in range(L)]
    arena = b.p3_arena_elems(plan)
    bf16 = grads[0].dtype == np.uint16
    gpad = np.uint16(0x7FC0) if bf16 else np.float32(np.nan)
    g = [to_device(sy.flat_to_arena(x, sizes, offs, arena, fill=gpad)) for x in grads]
    w = to_device(sy.flat_to_arena(w0, sizes, offs, arena, fill=PAD_W))
    m = to_device(sy.flat_to_arena(m0, sizes, offs, arena, fill=PAD_W))
    order = torch.full((K,), -1, dtype=torch.int32, device="cuda")
    result = torch.full((4,), -7, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    b.p3_drain_static(plan, [t.data_ptr() for t in g], b.P3_GRAD_BF16 if bf16 else b.P3_GRAD_FP32,
                      w.data_ptr(), m.data_ptr(), lr, mu, rescale, wd, marks, order.data_ptr(), result.data_ptr(),
                      stream.cuda_stream)
    stream.synchronize()
    wa, ma = w.cpu().numpy(), m.cpu().numpy()
    keep = np.ones(arena, dtype=bool)
    for n, o in zip(sizes, offs):
        keep[o:o + n] = False
    assert (wa[keep] == PAD_W).all() and (ma[keep] == PAD_W).all(), "padding was written"
    return (sy.arena_to_flat(wa, sizes, offs), sy.arena_to_flat(ma, sizes, offs), order.cpu().numpy(),
            result.cpu().numpy())


def run_bound(sizes, S, grads, w0, m0, marks, lr, mu, rescale, wd):
    case = DeviceCase(sizes, S, grads, w0, m0)
    b.p3_set_hyper(case.plan, lr, mu, rescale, wd)
    case.iterate(marks=marks, many=True)
    case.sync()
    w, m = case.fetch()
    return w, m, case.order()


def test_static_drain_equals_bound_drain_twice_in_a_row():
    stream = torch.cuda.Stream()
    rng = np.random.default_rng(20241)
    # first call: 40 ragged layers, 3 fp32 copies, weight decay and rescale in use, every layer marked
    sizes1 = [int(x) for x in rng.integers(1, 30000, size=37)] + [3328 * 5, 1, 7]
    S1 = 4096
    cfg1 = dict(seed=901, W=3, dtype="fp32", sigma_g=0.01, sigma_w=0.05, layers=sizes1)
    g1, w1, m1 = sy.make_inputs(cfg1)
    m1 = (0.01 * np.random.default_rng(5).standard_normal(m1.shape)).astype(np.float32)
    marks1 = list(range(len(sizes1) - 1, -1, -1))
    # second call, right behind it: smaller (9 layers), bf16 copies, only some layers marked, other order
    sizes2 = [5000, 64, 12345, 3, 800, 4097, 2, 30000, 11]
    S2 = 1000
    cfg2 = dict(seed=902, W=2, dtype="bf16", sigma_g=0.01, sigma_w=0.05, layers=sizes2)
    g2, w2, m2 = sy.make_inputs(cfg2)
    marks2 = [7, 2, 8, 0, 4]

    sw1, sm1, so1, sr1 = run_static(sizes1, S1, g1, w1, m1, marks1, 0.1, 0.9, 0.5, 1e-3, stream)
    sw2, sm2, so2, sr2 = run_static(sizes2, S2, g2, w2, m2, marks2, 0.05, 0.8, 1.0, 0.0, stream)

    bw1, bm1, bo1 = run_bound(sizes1, S1, g1, w1, m1, marks1, 0.1, 0.9, 0.5, 1e-3)
    bw2, bm2, bo2 = run_bound(sizes2, S2, g2, w2, m2, marks2, 0.05, 0.8, 1.0, 0.0)

    K1 = OraclePlan(sizes1, S1).K
    assert list(sr1) == [K1, 0, 0, len(sizes1)], sr1
    assert (so1 == bo1).all() and (so1 == np.arange(K1)).all()
    assert_same_bits(sw1, sm1, bw1, bm1, "static call 1 vs bound path")

    o2 = OraclePlan(sizes2, S2)
    want2 = o2.order_snapshot(marks2 + [-1])
    assert list(sr2) == [len(want2), 0, 0, len(marks2)], sr2
    assert (so2[:len(want2)] == bo2).all() and (bo2 == want2).all()
    assert (so2[len(want2):] == -1).all()                       # nothing logged beyond the claims
    assert_same_bits(sw2, sm2, bw2, bm2, "static call 2 vs bound path")
    # and the oracle, for the marked layers; unmarked layers untouched
    rw, rm = w2.copy(), m2.copy()
    o2.apply(want2, g2, rw, rm, 0.05, 0.8)
    assert_same_bits(sw2, sm2, rw, rm, "static call 2 vs oracle")


def test_static_drain_rejects_what_does_not_fit():
    lib = b.load()
    big = b.p3_plan([4096 * (b.P3_STATIC_MAX_SLICES + 1)], 4096)       # one slice too many
    many = b.p3_plan([8] * (b.P3_STATIC_MAX_LAYERS + 1), 4096)
    ok = b.p3_plan([64, 64], 4096)
    sharded = b.p3_plan_sharded([64, 64], 16, 2, 0)
    buf = torch.zeros(4096, dtype=torch.float32, device="cuda")
    out = torch.zeros(8192, dtype=torch.int32, device="cuda")

    def call(plan, marks, W=1):
        with pytest.raises(b.P3Error) as e:
            b.p3_drain_static(plan, [buf.data_ptr()] * W, b.P3_GRAD_FP32, buf.data_ptr(), buf.data_ptr(), 0.1, 0.9,
                              1.0, 0.0, marks, out.data_ptr(), out.data_ptr(), 0)
        return e.value.status

    assert call(big, [0]) == b.P3_ERR_RANGE
    assert call(many, [0]) == b.P3_ERR_RANGE
    assert call(ok, [0, 0]) == b.P3_ERR_ALREADY
    assert call(ok, [2]) == b.P3_ERR_RANGE
    assert call(sharded, [0]) == b.P3_ERR_ARG
    assert lib is not None
    torch.cuda.synchronize()
    assert (buf == 0).all()                                             # nothing was launched
