#!/usr/bin/env python3
"""Benchmark of the P3 parameter-server hot path on one MI355X.

One step = one synchronous-SGD iteration of the server: begin the iteration,
mark every layer ready in backward order (L-1 .. 0), drain (priority selection,
W-way aggregation, momentum + weight update, completion flags) -- all inputs
already resident in HBM.  Workload: the VGG-19-shaped parameter set, W = 8 fp32
gradient copies, slices of 50,000 parameters (paper Sec. 5.7), SGD momentum.

Prints ONE JSON line: aggregated-gradient GB/s (whole job), the HBM roofline of
the drain kernel measured with HIP events on the drain's stream (average, median
and minimum over the timed launches), per-iteration median and minimum from event
pairs, the layer-0 update latency in live mode, and the CPU oracle timed on the
host beside it.  The arenas lie where the library's own hint puts them
(p3_suggest_arena_stride); a probe of the naive placement is reported beside it.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


# HBM bytes per launch of the drain kernel from the FETCH_SIZE / WRITE_SIZE counter runs summarised in
# profiles/p3_drain_kernel_*_hbm_traffic.md (already scaled by what the counters read for a plain copy), valid
# for the kernel sources whose hash is given, the workload's default slice size and the default launch shape.
TRAFFIC = {
    "sources_sha256": "b624c4f9fec65e35dbe75ef78c1adb867aefcce31b194f9b3ba1f2da87426b7f",
    "bytes_per_launch": {"vgg19": 6901984589, "vgg19_bf16": 6902046605},
}


def kernel_source_hash():
    """sha256 over the kernel sources with comments and white space removed (so that only code changes count)."""
    import hashlib
    import re
    here = os.path.dirname(os.path.abspath(__file__))
    h = hashlib.sha256()
    for f in ("p3_drain.hip", "p3_internal.h", "p3_tiles.h"):
        with open(os.path.join(here, "paper_1905_03960_amd", "csrc", f), "r") as fh:
            text = fh.read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        text = re.sub(r"//[^\n]*", "", text)
        h.update(re.sub(r"\s+", "", text).encode())
    return h.hexdigest()


def measured_traffic(args, slice_elems, default_slice_elems):
    """Counter-measured HBM bytes per launch, or None once the kernel has changed since they were taken."""
    try:
        same_kernel = kernel_source_hash() == TRAFFIC["sources_sha256"]
    except OSError:
        return None
    same = (same_kernel and slice_elems == default_slice_elems and not args.tile_elems and not args.wgs_per_cu
            and not args.reserved_cus and args.shards == 1)
    return (TRAFFIC["bytes_per_launch"].get(args.workload) or None) if same else None


def stream_beside(torch, other, tries=16):
    """A new stream whose kernels run while a kernel of `other` is still running: HIP multiplexes streams over a
    few hardware queues, and two streams that share one are served one after the other (a live drain in front
    of its producer on such a pair would end by its watchdog).  Candidates are tried until one overlaps."""
    probe = torch.zeros(256, device="cuda")
    for _ in range(tries):
        cand = torch.cuda.Stream()
        busy, done = torch.cuda.Event(), torch.cuda.Event()
        torch.cuda.synchronize()
        with torch.cuda.stream(other):
            torch.cuda._sleep(60_000_000)
            busy.record(other)
        with torch.cuda.stream(cand):
            probe.add_(1)
            done.record(cand)
        done.synchronize()
        ok = not busy.query()
        torch.cuda.synchronize()
        if ok:
            return cand
    raise RuntimeError("no stream found that runs beside the drain's")


def overlap_study(b, torch, plan, sizes, stream, reps=5):
    """The drain beside a producer: one bf16 GEMM (rows x 4096 x 4096) per layer stands for the layer's
    backward step on a producer stream, and the layer is marked as that stream's next operation.  Ways to
    place the drain, each the best of `reps` iterations (ms from the first enqueue to the last update;
    device time from the selector seeing layer 0 to layer 0 being visible):
      serial        one snapshot drain on a second stream, after an event behind the last mark
      per_layer     a snapshot drain behind every mark (event + wait), so urgent layers go first among
                    whatever has been produced
      live_reserved one live drain launched before the backward, 64 compute units left to the producer
      live_lean     one live drain of the lean build (256-lane workgroups that share their compute unit)
                    launched before the backward, nothing reserved
    for four producers: GEMMs of 2048 and of 1536 rows (the library picks kernels with 128x256 and 128x192
    tiles for them, three quarters and half of a SIMD's register file per wavefront), one or two per layer (a
    backward step computes a data gradient and a weight gradient)."""
    L = len(sizes)
    producer = stream_beside(torch, stream)
    B = torch.randn(4096, 4096, device="cuda", dtype=torch.bfloat16)
    evs = [torch.cuda.Event() for _ in range(L)]

    def study(rows, per_layer, with_wide_live):
        A = torch.randn(rows, 4096, device="cuda", dtype=torch.bfloat16)
        C = torch.empty(rows, 4096, device="cuda", dtype=torch.bfloat16)

        def backward(mark, drain_each):
            for l in range(L - 1, -1, -1):
                with torch.cuda.stream(producer):
                    for _ in range(per_layer):
                        torch.matmul(A, B, out=C)
                    if mark:
                        b.p3_mark_ready_on_stream(plan, l, producer.cuda_stream)
                    if mark and (drain_each or l == 0):
                        evs[l].record(producer)
                        stream.wait_event(evs[l])
                        b.p3_drain(plan, stream.cuda_stream)

        def live():
            b.p3_drain(plan, stream.cuda_stream)
            for l in range(L - 1, -1, -1):
                with torch.cuda.stream(producer):
                    for _ in range(per_layer):
                        torch.matmul(A, B, out=C)
                    b.p3_mark_ready_on_stream(plan, l, producer.cuda_stream)

        def timed(fn, n=reps):
            best, lat = None, None
            for _ in range(n):
                b.p3_begin_iter(plan)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                fn()
                try:
                    b.p3_sync(plan, 10000)
                except b.P3Error as e:
                    torch.cuda.synchronize()
                    return {"ms": None, "note": f"the producer's kernels did not start beside the resident drain; "
                                                f"the drain's watchdog ended it ({e})"}
                torch.cuda.synchronize()
                t = (time.perf_counter() - t0) * 1e3
                if best is None or t < best:
                    best, lat = t, b.p3_layer_latency_ns(plan, 0)[1] / 1e3
            return {"ms": round(best, 3), "layer0_device_us": round(lat, 1)}

        def drain_alone():
            b.p3_profile_enable(plan, True)
            for _ in range(10):
                b.p3_begin_iter(plan)
                b.p3_mark_ready_many(plan, list(range(L - 1, -1, -1)))
                b.p3_drain(plan, stream.cuda_stream)
            b.p3_sync(plan)
            ms, n = b.p3_profile_read(plan)
            b.p3_profile_enable(plan, False)
            return round(ms / n, 4)

        res = {"producer": f"{L * per_layer} bf16 GEMMs {rows}x4096x4096, {per_layer} per layer, marks on the "
                           f"producer stream"}
        for _ in range(2):
            backward(False, False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            backward(False, False)
        torch.cuda.synchronize()
        res["backward_alone_ms"] = round((time.perf_counter() - t0) / reps * 1e3, 3)
        res["drain_alone_ms"] = drain_alone()
        res["serial"] = timed(lambda: backward(True, False))
        if with_wide_live:
            res["per_layer"] = timed(lambda: backward(True, True))
            b.p3_set_mode(plan, b.P3_MODE_LIVE)
            b.p3_set_reserved_cus(plan, 64)
            res["live_reserved"] = timed(live)
            b.p3_set_reserved_cus(plan, 0)
            b.p3_set_mode(plan, b.P3_MODE_SNAPSHOT)
        # the lean build: first alone (snapshot drains), then resident beside the backward pass
        b.p3_set_launch(plan, b.P3_LAUNCH_LEAN)
        res["lean_drain_alone_ms"] = drain_alone()
        b.p3_set_mode(plan, b.P3_MODE_LIVE)
        b.p3_set_tuning(plan, watchdog_ms=300)       # a producer that cannot start shows after 0.3 s
        first = timed(live, 1)
        res["live_lean"] = timed(live) if first["ms"] is not None else first
        b.p3_set_tuning(plan, watchdog_ms=10000)
        b.p3_set_mode(plan, b.P3_MODE_SNAPSHOT)
        b.p3_set_launch(plan, b.P3_LAUNCH_FUSED)
        if res["live_lean"]["ms"] is not None:
            res["live_lean"]["of_serial_sum"] = round(res["live_lean"]["ms"] /
                                                      (res["backward_alone_ms"] + res["drain_alone_ms"]), 3)
        return res

    return {"gemm_rows_2048": study(2048, 1, True), "gemm_rows_2048_two_per_layer": study(2048, 2, False),
            "gemm_rows_1536": study(1536, 1, False), "gemm_rows_1536_two_per_layer": study(1536, 2, False)}


def fixed_cost_study(b, torch, W=8, sizes_m=(24, 48, 96, 144), reps=12):
    """What a launch costs beyond the bytes it moves: one-layer fp32 parameter sets of several sizes (arenas at
    the suggested stride, one snapshot drain per iteration, kernel time from the library's HIP events), a
    straight line through (bytes, kernel time): the slope is the rate at which the kernel streams once it is
    under way, the intercept what every launch pays whatever its size (launch, first selection step, the last
    tiles running out)."""
    import numpy as np
    pts = []
    stream = torch.cuda.Stream()
    for m in sizes_m:
        n = m * 1000 * 1000
        plan = b.p3_plan([n], 50000)
        arena = b.p3_arena_elems(plan)
        slot = b.p3_suggest_arena_stride(plan, b.P3_GRAD_FP32)
        pool = torch.empty((W + 2) * slot + (1 << 21), dtype=torch.uint8, device="cuda")
        v = [pool[i * slot:i * slot + arena * 4].view(torch.float32) for i in range(W + 2)]
        for t in v[:W]:
            t.normal_(0, 1e-3)
        v[W].normal_(0, 0.05)
        v[W + 1].zero_()
        b.p3_bind(plan, [t.data_ptr() for t in v[:W]], b.P3_GRAD_FP32, v[W].data_ptr(), v[W + 1].data_ptr())
        b.p3_set_hyper(plan, 0.1, 0.9)
        for it in range(reps + 2):
            if it == 2:
                b.p3_sync(plan)
                b.p3_profile_enable(plan, True)
            b.p3_begin_iter(plan)
            b.p3_mark_ready(plan, 0)
            b.p3_drain(plan, stream.cuda_stream)
        ms, cnt = b.p3_profile_read(plan)
        b.p3_profile_enable(plan, False)
        pts.append(((W * 4 + 16) * n, ms / cnt))
        b.p3_destroy(plan)
        del v, pool
    x = np.array([p[0] for p in pts], dtype=np.float64)
    y = np.array([p[1] for p in pts], dtype=np.float64)
    slope, icpt = np.polyfit(x, y, 1)                 # ms per byte, ms
    rate = 1.0 / slope / 1e6                          # GB/s
    return {"what": f"one-layer fp32 sets, W={W}, kernel ms by HIP events, least-squares line",
            "points": [{"bytes": int(p[0]), "kernel_ms": round(p[1], 4)} for p in pts],
            "marginal_GBps": round(rate, 1), "marginal_frac": round(rate / HBM_PEAK_GBPS, 4),
            "fixed_us_per_launch": round(icpt * 1e3, 1)}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="vgg19",
                    choices=["mlp", "resnet50", "vgg19", "seq2seq", "vgg19_bf16"])
    ap.add_argument("--slice-elems", type=int, default=0)
    ap.add_argument("--tile-elems", type=int, default=0)
    ap.add_argument("--wgs-per-cu", type=int, default=0)
    ap.add_argument("--reserved-cus", type=int, default=0, help="compute units the drain leaves to other streams")
    ap.add_argument("--persistent", type=int, default=-1, help="1: one fused launch per drain, 0: selector + workers, 2: the lean build (256-lane workgroups that "
                         "share their compute unit)")
    ap.add_argument("--placement", default="suggested", choices=["suggested", "packed", "separate", "search", "best"],
                    help="where the arenas lie: at the distance p3_suggest_arena_stride gives (default), back to back, "
                         "in separate allocations; 'search' also probes other distances and reports them (the timed "
                         "run stays on the suggested one), 'best' times the fastest of them")
    ap.add_argument("--placement-trials", type=int, default=6, help="distances probed by --placement search/best")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy 3 times (reference for HBM byte counters)")
    ap.add_argument("--shards", type=int, default=1,
                    help="time one server's share: the plan owns the slices whose id is --shard modulo this number")
    ap.add_argument("--shard", type=int, default=0)
    ap.add_argument("--curves", action="store_true",
                    help="add 'layer_visible_us': when each layer's update became visible in the last live drain, "
                         "under the priority rule and under first-come-first-served")
    ap.add_argument("--overlap", action="store_true",
                    help="also time the drain beside a synthetic backward pass (bf16 GEMMs on a producer stream "
                         "that marks each layer as its next operation); adds an 'overlap' object to the line")
    ap.add_argument("--fixed-cost", action="store_true",
                    help="add 'fixed_cost': drains of one-layer sets of several sizes, the rate at which the kernel "
                         "streams once under way (slope) and what every launch pays whatever its size (intercept)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU only (the W workers are W gradient buffers in one "
              "GPU's HBM); --gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_1905_03960_amd import binding as b
    from paper_1905_03960_amd import synthetic as sy

    b.load()                       # fails loudly if libp3.so has not been built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)

    cfg = sy.config(args.workload)
    sizes = cfg["layers"]
    S = args.slice_elems or cfg["slice_elems"]
    W, bf16 = cfg["W"], cfg["dtype"] == "bf16"
    bg = 2 if bf16 else 4
    N = sum(sizes)

    t0 = time.time()
    plan = b.p3_plan_sharded(sizes, S, args.shards, args.shard) if args.shards > 1 else b.p3_plan(sizes, S)
    plan_us = (time.time() - t0) * 1e6
    L, K = len(sizes), b.p3_num_slices(plan)
    N_model, N = N, b.p3_num_elems(plan)          # the bytes below count what this plan owns
    owned = np.arange(args.shard, b.p3_shard_info(plan)[2], args.shards, dtype=np.int32)
    offs = [b.p3_layer_offset(plan, l) for l in range(L)]
    arena = b.p3_arena_elems(plan)

    grads, w0, m0 = sy.make_inputs(cfg, threads=min(16, os.cpu_count() or 1))
    dtype_code = b.P3_GRAD_BF16 if bf16 else b.P3_GRAD_FP32
    per = (arena * 4 + (1 << 21) - 1) // (1 << 21) * (1 << 21)              # an arena rounded up to 2 MiB
    held = []                                                                 # device allocations alive

    def release(pl):
        held[:] = [x for x in held if x is not pl["pool"]]
        pl["pool"], pl["views"] = None, None

    def place(slot, src=None):
        """All W + 2 arenas in one fresh allocation, `slot` bytes apart (slot < 0: separate allocations).
        Data comes from the host (src None) or from another placement's views (copied on the device)."""
        pool = None if slot < 0 else torch.empty((W + 2) * slot + (1 << 21), dtype=torch.uint8, device="cuda")
        views = []
        for i in range(W + 2):
            if src is None:
                a = grads[i] if i < W else (w0 if i == W else m0)
                x = sy.flat_to_arena(a, sizes, offs, arena)
                t = torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x)
            else:
                t = src[i]
            if pool is None:
                views.append(t.cuda() if src is None else t.clone())
            else:
                nbytes = t.numel() * t.element_size()
                v = pool[i * slot:i * slot + nbytes].view(t.dtype)
                v.copy_(t)
                views.append(v)
        torch.cuda.synchronize()
        if pool is not None:
            held.append(pool)
        return {"slot": slot, "pool": pool, "views": views}

    def bind(pl):
        v = pl["views"]
        b.p3_bind(plan, [t.data_ptr() for t in v[:W]], dtype_code, v[W].data_ptr(), v[W + 1].data_ptr())

    stream = torch.cuda.Stream()
    if args.tile_elems or args.wgs_per_cu:
        b.p3_set_tuning(plan, args.tile_elems, args.wgs_per_cu, 0, 0)
    if args.reserved_cus:
        b.p3_set_reserved_cus(plan, args.reserved_cus)
    order = list(range(L - 1, -1, -1))

    def step():
        b.p3_begin_iter(plan)
        b.p3_mark_ready_many(plan, order)
        b.p3_drain(plan, stream.cuda_stream)

    def probe(pl, n=10):
        """Median kernel time of n drains on a placement (after three untimed ones)."""
        bind(pl)
        for _ in range(3):
            step()
        b.p3_sync(plan)
        b.p3_profile_enable(plan, True)
        for _ in range(n):
            step()
        _, _, each = b.p3_profile_read(plan, each=n)
        b.p3_profile_enable(plan, False)
        return float(np.median(each))

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    # Where the arenas lie moves the rate by several per cent.  The timed run uses the placement the library
    # itself suggests (p3_suggest_arena_stride: one allocation, a fixed distance between the arenas), with no
    # search.  Beside it the line reports a short probe of the naive placement (arenas back to back), and with
    # --placement search a few other spacings are probed as well (one candidate at a time: never more than
    # two placements are alive), without changing what is timed unless --placement best is given.
    suggested = b.p3_suggest_arena_stride(plan, dtype_code)
    first_slot = {"suggested": suggested, "packed": per, "separate": -1}.get(args.placement, suggested)
    if args.placement in ("search", "best"):
        first_slot = suggested
    chosen = place(first_slot)
    bind(chosen)
    b.p3_set_hyper(plan, cfg["lr"], cfg["mu"])
    if args.persistent >= 0:
        b.p3_set_launch(plan, args.persistent)
    placement = {"mode": args.placement, "suggested_slot_MiB": round(suggested / 2 ** 20, 1),
                 "timed_slot_MiB": round(first_slot / 2 ** 20, 1) if first_slot > 0 else "separate allocations"}
    big = arena * 4 >= (64 << 20)                       # a probe is pointless for tiny models
    if big and args.placement != "packed" and torch.cuda.mem_get_info()[0] > (W + 2) * per + (8 << 30):
        for _ in range(20):                              # the first drains of a process run slower than the rest:
            step()                                       # none of them goes into a probe
        b.p3_sync(plan)
        timed_probe = probe(chosen)
        packed = place(per, chosen["views"])
        packed_ms = probe(packed)
        placement["probe_kernel_ms"] = {"timed_placement": round(timed_probe, 4), "packed": round(packed_ms, 4)}
        placement["packed_frac"] = round((W * bg + 16) * N / (packed_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)
        trials = []
        if args.placement in ("search", "best"):
            gib = 1 << 30
            unit = (arena * 4 + (256 << 20) - 1) // (256 << 20) * (256 << 20)
            slots = [gib * ((arena * 4 + gib - 1) // gib), unit, unit + (256 << 20), 2 * gib, 2 * gib + (256 << 20),
                     2 * gib + (512 << 20), unit + (512 << 20), 3 * gib]
            slots = [x for i, x in enumerate(slots) if x >= arena * 4 and x not in slots[:i] and x != suggested
                     and x != per][:args.placement_trials]
            best, best_ms = chosen, timed_probe
            release(packed)                                # its probe is on record
            for slot in slots:
                if torch.cuda.mem_get_info()[0] < (W + 2) * slot + (4 << 30):
                    continue
                cand = place(slot, best["views"])
                ms = probe(cand)
                trials.append({"slot_MiB": round(slot / 2 ** 20, 1), "probe_kernel_ms": round(ms, 4)})
                loser = cand if ms >= best_ms else best
                if ms < best_ms:
                    best, best_ms = cand, ms
                release(loser)
            placement["trials"] = trials
            placement["best_slot_MiB"] = round(best["slot"] / 2 ** 20, 1)
            if args.placement == "best":
                chosen = best
                placement["timed_slot_MiB"] = placement["best_slot_MiB"]
            elif best is not chosen:
                chosen = place(suggested, best["views"])
                release(best)
            # released device memory is cleared by the driver in the background, which was measured to slow
            # the drains that follow by 1 % for a few seconds: wait that out before the timed region
            torch.cuda.synchronize()
            time.sleep(4.0)
        bind(chosen)
        placement["held_GiB"] = round(sum(x.numel() for x in held) / 2 ** 30, 1)
    g, w, m = chosen["views"][:W], chosen["views"][W], chosen["views"][W + 1]

    for _ in range(args.warmup):
        step()
    b.p3_sync(plan)
    torch.cuda.synchronize()

    # Timed region: K iterations back to back (whole-job rate); the drain kernel of each is bracketed by the
    # library's own HIP event pair on the drain's stream (roofline: average, median, minimum).
    b.p3_profile_enable(plan, True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    b.p3_sync(plan)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kern_ms, launches, kern_each = b.p3_profile_read(plan, each=args.steps)
    sel_first_ns, sel_done_ns = b.p3_selector_timeline_ns(plan)
    b.p3_profile_enable(plan, False)
    claimed = b.p3_query_order(plan)
    assert claimed.shape[0] == K and (claimed == owned).all(), "drain did not claim every slice in order"
    # A second pass of K iterations, each between its own pair of HIP events on the drain's stream: median and
    # minimum per iteration (the events themselves cost about 10 us per iteration, so this pass is not the
    # one the whole-job rate is taken from).
    ev0 = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    ev1 = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    for i in range(args.steps):
        ev0[i].record(stream)
        step()
        ev1[i].record(stream)
    b.p3_sync(plan)
    torch.cuda.synchronize()
    iter_each = np.array([a.elapsed_time(c) for a, c in zip(ev0, ev1)])

    ms_per_step = elapsed / args.steps * 1e3
    agg_gbps = W * N * bg / (elapsed / args.steps) / 1e9
    bytes_per_launch = (W * bg + 16) * N           # W gradient reads + w,m read + w,m write per parameter
    kern_avg_ms = kern_ms / max(launches, 1)
    achieved = bytes_per_launch / (kern_avg_ms * 1e-3) / 1e9

    # layer-0 update latency: live drain running while layers are marked L-1 .. 0
    b.p3_set_mode(plan, b.P3_MODE_LIVE)
    lat_host, lat_dev = [], []
    for _ in range(5):
        b.p3_begin_iter(plan)
        b.p3_drain(plan, stream.cuda_stream)
        for l in order:
            b.p3_mark_ready(plan, l)
        b.p3_wait_layer(plan, 0, 10000)
        b.p3_sync(plan, 10000)
        h, d = b.p3_layer_latency_ns(plan, 0)
        lat_host.append(h / 1e3)
        lat_dev.append(d / 1e3)
    curve_priority = [round(b.p3_layer_timeline_ns(plan, l)[1] / 1e3, 1) for l in range(L)] if args.curves else None
    # The drain as a training loop would run it: launched at the start of the iteration, resident and waiting
    # when the gradients arrive.  Here all layers are marked at once 0.3 ms after the launch; the time runs
    # on the device clock from the first mark the selector sees to the last layer's update being visible.
    resident_ms = []
    for _ in range(7):
        b.p3_begin_iter(plan)
        b.p3_drain(plan, stream.cuda_stream)
        time.sleep(0.0003)
        b.p3_mark_ready_many(plan, order)
        b.p3_sync(plan, 10000)
        stamps = [b.p3_layer_timeline_ns(plan, l) for l in range(L)]
        resident_ms.append((max(d for _, d in stamps) - min(sn for sn, _ in stamps)) / 1e6)
    # the same with the first-come-first-served baseline (layers whole, in mark order): layer 0, marked last,
    # waits behind everything marked before it
    b.p3_set_policy(plan, b.P3_POLICY_FIFO)
    fifo_host, fifo_dev = [], []
    for _ in range(3):
        b.p3_begin_iter(plan)
        b.p3_drain(plan, stream.cuda_stream)
        for l in order:
            b.p3_mark_ready(plan, l)
        b.p3_wait_layer(plan, 0, 10000)
        b.p3_sync(plan, 10000)
        h, d = b.p3_layer_latency_ns(plan, 0)
        fifo_host.append(h / 1e3)
        fifo_dev.append(d / 1e3)
    curve_fifo = [round(b.p3_layer_timeline_ns(plan, l)[1] / 1e3, 1) for l in range(L)] if args.curves else None
    b.p3_set_policy(plan, b.P3_POLICY_PRIORITY)
    b.p3_set_mode(plan, b.P3_MODE_SNAPSHOT)

    out = {
        "metric": "aggregated gradient GB/s (fraction of HBM peak); layer-0 update latency",
        "value": round(agg_gbps, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_iteration_events": {"median": round(float(np.median(iter_each)), 4), "min": round(float(iter_each.min()), 4),
                                "note": "second pass of the same K iterations, one HIP event pair per iteration"},
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16-in/f32" if bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": (f"share {args.shard} of {args.shards} (slices round robin, {N} parameters owned) of "
                                if args.shards > 1 else "") +
                               f"{args.workload}: {L} tensors, {N_model} params, W={W} {cfg['dtype']} gradient copies, "
                               f"slice_elems={S} ({K} slices), SGD lr={cfg['lr']} momentum={cfg['mu']}, "
                               f"marks {L - 1}..0 then one snapshot drain per iteration"},
        "hbm_GBps": round((W * bg + 16) * N / (elapsed / args.steps) / 1e9, 2),
        "hbm_frac": round((W * bg + 16) * N / (elapsed / args.steps) / 1e9 / HBM_PEAK_GBPS, 4),
        "layer0_latency_us": {"mode": "live, marks L-1..0 back to back", "host_median": round(float(np.median(lat_host)), 2),
                              "host_min": round(float(min(lat_host)), 2),
                              "device_median": round(float(np.median(lat_dev)), 2),
                              "fifo_policy_host_median": round(float(np.median(fifo_host)), 2),
                              "fifo_policy_device_median": round(float(np.median(fifo_dev)), 2)},
        "resident_drain": {"mode": "live drain launched 0.3 ms before the gradients, all layers marked at once; "
                                   "device clock, first mark seen -> last layer visible",
                           "ms_median": round(float(np.median(resident_ms)), 4), "ms_min": round(float(min(resident_ms)), 4),
                           "hbm_frac_median": round(bytes_per_launch / (float(np.median(resident_ms)) * 1e-3) / 1e9
                                                    / HBM_PEAK_GBPS, 4)},
        "plan_us": round(plan_us, 1),
        "placement": placement,
        "selector_us": {"first_publication": round(sel_first_ns / 1e3, 2), "finished": round(sel_done_ns / 1e3, 2)},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": measured_traffic(args, S, cfg["slice_elems"]),
                     "kernel": "p3_drain_kernel", "kernel_avg_ms": round(kern_avg_ms, 4),
                     "kernel_median_ms": round(float(np.median(kern_each)), 4),
                     "kernel_min_ms": round(float(kern_each.min()), 4), "launches": launches,
                     "bytes_per_launch": bytes_per_launch},
    }

    if args.curves:
        # when each layer's update is visible, on the device clock of the last live drain of each policy
        # (0 = the selector's first instruction; the layers are marked L-1..0 within the first microseconds)
        out["layer_visible_us"] = {"priority": curve_priority, "fifo_policy": curve_fifo}
    if args.overlap:
        out["overlap"] = overlap_study(b, torch, plan, sizes, stream)
    if args.fixed_cost:
        out["fixed_cost"] = fixed_cost_study(b, torch)

    if not args.no_cpu_baseline:
        import oracle
        o = oracle.OraclePlan(sizes, S)
        ident = owned
        cw, cm = w0.copy(), m0.copy()
        iters, t_cpu = 0, 0.0
        while iters < args.steps and (iters == 0 or t_cpu + t_cpu / iters <= args.cpu_seconds):
            t1 = time.perf_counter()
            o.apply(ident, grads, cw, cm, cfg["lr"], cfg["mu"])
            t_cpu += time.perf_counter() - t1
            iters += 1
        out["cpu_baseline"] = {"value": round(W * N * bg * iters / t_cpu / 1e9, 3), "unit": "GB/s", "cores": 1,
                               "kind": "oracle",
                               "sample": f"{iters} full iteration(s) of the same workload, {t_cpu:.1f} s, "
                                         f"single-threaded C++ oracle (g++ -O2 -ffp-contract=off)",
                               "host_cpus_visible": os.cpu_count()}
        # the same oracle on all host cores the process may use: slices split statically over T threads
        # (every element is independent, so the result is the same bits)
        from concurrent.futures import ThreadPoolExecutor
        T = max(1, min(16, len(os.sched_getaffinity(0))))
        chunks = [c for c in np.array_split(ident, T) if c.size]
        iters_t, t_thr = 0, 0.0
        with ThreadPoolExecutor(max_workers=T) as ex:
            while iters_t < args.steps and (iters_t == 0 or t_thr + t_thr / iters_t <= args.cpu_seconds / 2):
                t1 = time.perf_counter()
                list(ex.map(lambda c: o.apply(c, grads, cw, cm, cfg["lr"], cfg["mu"]), chunks))
                t_thr += time.perf_counter() - t1
                iters_t += 1
        out["cpu_baseline_threaded"] = {"value": round(W * N * bg * iters_t / t_thr / 1e9, 3), "unit": "GB/s",
                                        "cores": len(chunks), "kind": "oracle",
                                        "sample": f"{iters_t} full iteration(s), {t_thr:.1f} s, slices split "
                                                  f"statically over {len(chunks)} threads"}
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
