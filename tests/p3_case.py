"""Shared scaffolding of the GPU parity tests: puts seeded inputs into device
arenas (torch is used for device memory and streams only), drives the C-ABI
through the binding, and fetches results back into the oracle's flat layout."""
import numpy as np
import torch

from paper_1905_03960_amd import binding as b
from paper_1905_03960_amd import synthetic as sy

PAD_W = np.float32(12345.0)       # sentinel in weight/momentum padding: must survive
PAD_G = np.float32(np.nan)        # gradient padding: must never be read into a result


def stream_beside(*others, tries=16):
    """A new stream whose kernels run while kernels of `others` are still running.  HIP multiplexes its streams
    over a few hardware queues (four by default), and two streams that share a queue are served one after the
    other: a live drain launched in front of its producer on such a pair would wait for marks that cannot be
    made until it has ended.  Which streams share a queue is not documented, so candidates are tried."""
    probe = torch.zeros(256, device="cuda")
    for _ in range(tries):
        cand = torch.cuda.Stream()
        ok = True
        for other in others:
            busy, done = torch.cuda.Event(), torch.cuda.Event()
            torch.cuda.synchronize()
            with torch.cuda.stream(other):
                torch.cuda._sleep(60_000_000)            # tens of milliseconds
                busy.record(other)
            with torch.cuda.stream(cand):
                probe.add_(1)
                done.record(cand)
            done.synchronize()
            ok = ok and not busy.query()                # the candidate's kernel finished while the other still spins
            torch.cuda.synchronize()
        if ok:
            return cand
    raise RuntimeError("no stream found that runs beside the given ones")


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def to_device(arr):
    """numpy (float32 or uint16) -> device tensor holding the same bytes."""
    if arr.dtype == np.uint16:
        return torch.from_numpy(arr.view(np.int16)).cuda()
    return torch.from_numpy(arr).cuda()


class DeviceCase:
    def __init__(self, sizes, slice_elems, grads, w0, m0, tile_elems=0, wgs_per_cu=0,
                 lookahead=0, watchdog_ms=0, stream=None):
        self.sizes = [int(x) for x in sizes]
        self.plan = b.p3_plan(self.sizes, slice_elems)
        self.L = len(self.sizes)
        self.K = b.p3_num_slices(self.plan)
        self.offsets = [b.p3_layer_offset(self.plan, l) for l in range(self.L)]
        self.arena = b.p3_arena_elems(self.plan)
        self.bf16 = grads[0].dtype == np.uint16
        gpad = np.uint16(0x7FC0) if self.bf16 else PAD_G        # bf16 NaN pattern
        self.g = [to_device(sy.flat_to_arena(g, self.sizes, self.offsets, self.arena, fill=gpad)) for g in grads]
        self.w = to_device(sy.flat_to_arena(w0, self.sizes, self.offsets, self.arena, fill=PAD_W))
        self.m = to_device(sy.flat_to_arena(m0, self.sizes, self.offsets, self.arena, fill=PAD_W))
        self.stream = stream if stream is not None else torch.cuda.Stream()
        torch.cuda.synchronize()
        if tile_elems or wgs_per_cu or lookahead or watchdog_ms:
            b.p3_set_tuning(self.plan, tile_elems, wgs_per_cu, lookahead, watchdog_ms)
        b.p3_bind(self.plan, [t.data_ptr() for t in self.g],
                  b.P3_GRAD_BF16 if self.bf16 else b.P3_GRAD_FP32, self.w.data_ptr(), self.m.data_ptr())

    # one iteration in snapshot mode: marks (reverse layer order by default), then one drain
    def iterate(self, marks=None, drain_each=False, many=False):
        marks = list(range(self.L - 1, -1, -1)) if marks is None else marks
        b.p3_begin_iter(self.plan)
        if many:                                   # one call for all marks
            b.p3_mark_ready_many(self.plan, marks)
            marks = []
        for l in marks:
            b.p3_mark_ready(self.plan, l)
            if drain_each:
                b.p3_drain(self.plan, self.stream.cuda_stream)
        if not drain_each:
            b.p3_drain(self.plan, self.stream.cuda_stream)

    def sync(self, timeout_ms=-1):
        b.p3_sync(self.plan, timeout_ms)

    def order(self):
        return b.p3_query_order(self.plan)

    def fetch(self):
        """(w, m) in the flat unpadded layout, plus a check that padding is untouched."""
        self.stream.synchronize()
        wa, ma = self.w.cpu().numpy(), self.m.cpu().numpy()
        keep = np.ones(self.arena, dtype=bool)
        for n, o in zip(self.sizes, self.offsets):
            keep[o:o + n] = False
        assert (wa[keep] == PAD_W).all() and (ma[keep] == PAD_W).all(), "padding was written"
        return sy.arena_to_flat(wa, self.sizes, self.offsets), sy.arena_to_flat(ma, self.sizes, self.offsets)


def assert_same_bits(got_w, got_m, ref_w, ref_m, what=""):
    dw = int((bits(got_w) != bits(ref_w)).sum())
    dm = int((bits(got_m) != bits(ref_m)).sum())
    assert dw == 0 and dm == 0, f"{what}: {dw} weight and {dm} momentum elements differ in bits"
