"""ctypes binding of the C-ABI library declared in include/p3.h.

Argument marshalling only: every step of the hot path (slice table, selection,
aggregation, update, completion flags) runs inside libp3.so.  Device memory is
whatever the caller allocated (e.g. torch tensors; pass `tensor.data_ptr()`),
streams are raw hipStream_t values (`torch.cuda.Stream().cuda_stream`).

The library is opened on first use.  If it has not been built the import of a
symbol fails loudly; there is no fallback implementation.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libp3.so")

P3_OK = 0
P3_ERR_ARG, P3_ERR_STATE, P3_ERR_RANGE, P3_ERR_ALREADY = -1, -2, -3, -4
P3_ERR_NOMEM, P3_ERR_DEVICE, P3_ERR_TIMEOUT, P3_ERR_INCOMPLETE = -5, -6, -7, -8
P3_GRAD_FP32, P3_GRAD_BF16 = 0, 1
P3_MODE_SNAPSHOT, P3_MODE_LIVE, P3_MODE_TICKED = 0, 1, 2
P3_POLICY_PRIORITY, P3_POLICY_FIFO = 0, 1
P3_LAUNCH_SPLIT, P3_LAUNCH_FUSED, P3_LAUNCH_LEAN = 0, 1, 2
P3_MAX_WORKERS = 64
P3_STATIC_MAX_LAYERS, P3_STATIC_MAX_SLICES = 256, 4096

_vp, _i32, _i64, _f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
_P = C.POINTER

# name -> (restype, argtypes): exactly the declarations of include/p3.h
SIGNATURES = {
    "p3_plan": (C.c_int, [_P(_i64), _i32, _i64, _P(_vp)]),
    "p3_plan_sharded": (C.c_int, [_P(_i64), _i32, _i64, _i32, _i32, _P(_vp)]),
    "p3_shard_info": (C.c_int, [_vp, _P(_i32), _P(_i32), _P(_i32)]),
    "p3_slice_global_id": (_i32, [_vp, _i32]),
    "p3_destroy": (None, [_vp]),
    "p3_num_layers": (_i32, [_vp]),
    "p3_num_slices": (_i32, [_vp]),
    "p3_num_elems": (_i64, [_vp]),
    "p3_arena_elems": (_i64, [_vp]),
    "p3_layer_offset": (_i64, [_vp, _i32]),
    "p3_layer_first_slice": (_i32, [_vp, _i32]),
    "p3_layer_num_slices": (_i32, [_vp, _i32]),
    "p3_slice_info": (C.c_int, [_vp, _i32, _P(_i32), _P(_i64), _P(_i32)]),
    "p3_suggest_arena_stride": (_i64, [_vp, _i32]),
    "p3_bind": (C.c_int, [_vp, _i32, _P(_vp), _i32, _vp, _vp]),
    "p3_set_hyper": (C.c_int, [_vp, _f32, _f32, _f32, _f32]),
    "p3_set_mode": (C.c_int, [_vp, _i32, _P(_i64)]),
    "p3_set_tuning": (C.c_int, [_vp, _i32, _i32, _i32, _i32]),
    "p3_set_launch": (C.c_int, [_vp, _i32]),
    "p3_set_reserved_cus": (C.c_int, [_vp, _i32]),
    "p3_set_policy": (C.c_int, [_vp, _i32]),
    "p3_begin_iter": (C.c_int, [_vp]),
    "p3_mark_ready": (C.c_int, [_vp, _i32]),
    "p3_mark_ready_many": (C.c_int, [_vp, C.POINTER(C.c_int32), _i32]),
    "p3_wait_layer_on_stream": (C.c_int, [_vp, _i32, _vp, _i32]),
    "p3_stream_wait_expired": (C.c_int, [_vp]),
    "p3_mark_ready_on_stream": (C.c_int, [_vp, _i32, _vp]),
    "p3_drain": (C.c_int, [_vp, _vp]),
    "p3_sync": (C.c_int, [_vp, _i32]),
    "p3_poll": (C.c_int, [_vp]),
    "p3_abort": (C.c_int, [_vp]),
    "p3_wait_layer": (C.c_int, [_vp, _i32, _i32]),
    "p3_query_order": (_i32, [_vp, _P(_i32), _i32]),
    "p3_query_trace": (_i32, [_vp, _P(_i32), _i32]),
    "p3_layer_latency_ns": (C.c_int, [_vp, _i32, _P(_i64), _P(_i64)]),
    "p3_layer_timeline_ns": (C.c_int, [_vp, _i32, _P(_i64), _P(_i64)]),
    "p3_drain_status": (C.c_int, [_vp, _P(_i32), _P(_i32), _P(_i32), _P(_i32)]),
    "p3_selector_timeline_ns": (C.c_int, [_vp, _P(_i64), _P(_i64)]),
    "p3_profile_enable": (C.c_int, [_vp, _i32]),
    "p3_profile_read": (C.c_int, [_vp, _P(C.c_double), _P(_i32), _P(C.c_float), _i32]),
    "p3_drain_static": (C.c_int, [_vp, _i32, _P(_vp), _i32, _vp, _vp, _f32, _f32, _f32, _f32, _P(_i32), _i32, _vp, _vp,
                                  _vp]),
    "p3_last_hip_error": (C.c_int, [_P(C.c_int)]),
    "p3_strerror": (C.c_char_p, [C.c_int]),
}

_lib = None


def load():
    """Open libp3.so and declare every entry point.  Raises if it is not built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1905_03960_amd.build` "
                "(there is no fallback path)")
        # PyTorch bundles its own HIP runtime.  It has to be in the process before
        # libp3.so is opened, so that libp3 binds to that same runtime: a second
        # runtime loaded beside it cannot use the device torch's tensors live on.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


class P3Error(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = f"{where}: {strerror(status)} ({status})"
        if status == P3_ERR_DEVICE:
            code, line = p3_last_hip_error()
            msg += f" [hipError {code} at runtime source line {line}]"
        super().__init__(msg)


def p3_last_hip_error():
    line = C.c_int()
    code = load().p3_last_hip_error(C.byref(line))
    return code, line.value


def strerror(status):
    return load().p3_strerror(int(status)).decode()


def _check(status, where):
    if status != P3_OK:
        raise P3Error(status, where)


def _h(plan):
    return plan.handle if isinstance(plan, Plan) else plan


class Plan:
    """Owner of a p3_plan_t* (destroyed with the object)."""

    def __init__(self, handle):
        self.handle = handle

    def __del__(self):
        h, self.handle = getattr(self, "handle", None), None
        if h and _lib is not None:
            _lib.p3_destroy(h)


# ---- the calls, same names as the C ABI --------------------------------------
def p3_plan(layer_sizes, slice_elems):
    sizes = np.ascontiguousarray(layer_sizes, dtype=np.int64)
    out = _vp()
    _check(load().p3_plan(sizes.ctypes.data_as(_P(_i64)), int(sizes.shape[0]), int(slice_elems), C.byref(out)),
           "p3_plan")
    return Plan(out.value)


def p3_plan_sharded(layer_sizes, slice_elems, n_shards, shard):
    sizes = np.ascontiguousarray(layer_sizes, dtype=np.int64)
    out = _vp()
    _check(load().p3_plan_sharded(sizes.ctypes.data_as(_P(_i64)), int(sizes.shape[0]), int(slice_elems),
                                  int(n_shards), int(shard), C.byref(out)), "p3_plan_sharded")
    return Plan(out.value)


def p3_shard_info(plan):
    n, j, k = _i32(), _i32(), _i32()
    _check(load().p3_shard_info(_h(plan), C.byref(n), C.byref(j), C.byref(k)), "p3_shard_info")
    return n.value, j.value, k.value


def p3_slice_global_id(plan, g):
    r = load().p3_slice_global_id(_h(plan), int(g))
    if r < 0:
        _check(r, "p3_slice_global_id")
    return r


def p3_destroy(plan):
    if isinstance(plan, Plan):
        h, plan.handle = plan.handle, None
    else:
        h = plan
    if h:
        load().p3_destroy(h)


def p3_num_layers(plan):
    return load().p3_num_layers(_h(plan))


def p3_num_slices(plan):
    return load().p3_num_slices(_h(plan))


def p3_num_elems(plan):
    return load().p3_num_elems(_h(plan))


def p3_arena_elems(plan):
    return load().p3_arena_elems(_h(plan))


def p3_layer_offset(plan, layer):
    return load().p3_layer_offset(_h(plan), int(layer))


def p3_layer_first_slice(plan, layer):
    return load().p3_layer_first_slice(_h(plan), int(layer))


def p3_layer_num_slices(plan, layer):
    return load().p3_layer_num_slices(_h(plan), int(layer))


def p3_slice_info(plan, g):
    layer, off, ln = _i32(), _i64(), _i32()
    _check(load().p3_slice_info(_h(plan), int(g), C.byref(layer), C.byref(off), C.byref(ln)), "p3_slice_info")
    return layer.value, off.value, ln.value


def p3_suggest_arena_stride(plan, grad_dtype):
    r = load().p3_suggest_arena_stride(_h(plan), int(grad_dtype))
    if r < 0:
        _check(int(r), "p3_suggest_arena_stride")
    return int(r)


def p3_bind(plan, grad_ptrs, grad_dtype, weights_ptr, momentum_ptr):
    """grad_ptrs: W device addresses (ints); weights_ptr/momentum_ptr: device addresses."""
    arr = (_vp * len(grad_ptrs))(*[int(p) for p in grad_ptrs])
    _check(load().p3_bind(_h(plan), len(grad_ptrs), arr, int(grad_dtype), _vp(int(weights_ptr)),
                          _vp(int(momentum_ptr))), "p3_bind")


def p3_set_hyper(plan, lr, mu, rescale=1.0, wd=0.0):
    _check(load().p3_set_hyper(_h(plan), float(lr), float(mu), float(rescale), float(wd)), "p3_set_hyper")


def p3_set_mode(plan, mode, release_tick=None):
    if release_tick is None:
        _check(load().p3_set_mode(_h(plan), int(mode), None), "p3_set_mode")
    else:
        r = np.ascontiguousarray(release_tick, dtype=np.int64)
        if r.shape != (p3_num_layers(plan),):
            raise ValueError("release_tick needs one entry per layer")
        _check(load().p3_set_mode(_h(plan), int(mode), r.ctypes.data_as(_P(_i64))), "p3_set_mode")


def p3_set_tuning(plan, tile_elems=0, wgs_per_cu=0, lookahead_tiles=0, watchdog_ms=0):
    _check(load().p3_set_tuning(_h(plan), int(tile_elems), int(wgs_per_cu), int(lookahead_tiles),
                                int(watchdog_ms)), "p3_set_tuning")


def p3_set_policy(plan, policy):
    _check(load().p3_set_policy(_h(plan), int(policy)), "p3_set_policy")


def p3_set_reserved_cus(plan, n_cus):
    _check(load().p3_set_reserved_cus(_h(plan), int(n_cus)), "p3_set_reserved_cus")


def p3_set_launch(plan, persistent):
    _check(load().p3_set_launch(_h(plan), int(persistent)), "p3_set_launch")


def p3_begin_iter(plan):
    _check(load().p3_begin_iter(_h(plan)), "p3_begin_iter")


def p3_mark_ready(plan, layer):
    _check(load().p3_mark_ready(_h(plan), int(layer)), "p3_mark_ready")


def p3_mark_ready_many(plan, layers):
    arr = (C.c_int32 * len(layers))(*[int(l) for l in layers])
    _check(load().p3_mark_ready_many(_h(plan), arr, len(layers)), "p3_mark_ready_many")


def p3_mark_ready_on_stream(plan, layer, stream):
    _check(load().p3_mark_ready_on_stream(_h(plan), int(layer), C.c_void_p(int(stream) if stream else None)),
           "p3_mark_ready_on_stream")


def p3_wait_layer_on_stream(plan, layer, stream, timeout_ms=-1):
    _check(load().p3_wait_layer_on_stream(_h(plan), int(layer), C.c_void_p(int(stream) if stream else None),
                                          int(timeout_ms)), "p3_wait_layer_on_stream")


def p3_stream_wait_expired(plan):
    rc = load().p3_stream_wait_expired(_h(plan))
    if rc < 0:
        _check(rc, "p3_stream_wait_expired")
    return bool(rc)


def p3_drain(plan, stream=0):
    _check(load().p3_drain(_h(plan), _vp(int(stream))), "p3_drain")


def p3_drain_static(plan, grad_ptrs, grad_dtype, weights_ptr, momentum_ptr, lr, mu, rescale, wd, ready_layers,
                    order_out_ptr, result_out_ptr, stream=0):
    """The allocation-free iteration: device addresses in, kernels enqueued on `stream`, nothing waited for."""
    arr = (_vp * len(grad_ptrs))(*[int(p) for p in grad_ptrs])
    lay = (C.c_int32 * max(len(ready_layers), 1))(*[int(l) for l in ready_layers])
    _check(load().p3_drain_static(_h(plan), len(grad_ptrs), arr, int(grad_dtype), _vp(int(weights_ptr)),
                                  _vp(int(momentum_ptr)), float(lr), float(mu), float(rescale), float(wd), lay,
                                  len(ready_layers), _vp(int(order_out_ptr)), _vp(int(result_out_ptr)),
                                  _vp(int(stream))), "p3_drain_static")


def p3_sync(plan, timeout_ms=-1):
    _check(load().p3_sync(_h(plan), int(timeout_ms)), "p3_sync")


def p3_poll(plan):
    """True once every issued drain has finished (non-blocking)."""
    rc = load().p3_poll(_h(plan))
    if rc == P3_ERR_TIMEOUT:
        return False
    _check(rc, "p3_poll")
    return True


def p3_abort(plan):
    _check(load().p3_abort(_h(plan)), "p3_abort")


def p3_wait_layer(plan, layer, timeout_ms=-1):
    _check(load().p3_wait_layer(_h(plan), int(layer), int(timeout_ms)), "p3_wait_layer")


def _log(fn, plan, where):
    cap = p3_num_slices(plan)
    out = np.empty(cap, dtype=np.int32)
    n = fn(_h(plan), out.ctypes.data_as(_P(_i32)), cap)
    if n < 0:
        raise P3Error(n, where)
    return out[:n].copy()


def p3_query_order(plan):
    return _log(load().p3_query_order, plan, "p3_query_order")


def p3_query_trace(plan):
    return _log(load().p3_query_trace, plan, "p3_query_trace")


def p3_layer_timeline_ns(plan, layer):
    seen, done = C.c_int64(0), C.c_int64(0)
    _check(load().p3_layer_timeline_ns(_h(plan), int(layer), C.byref(seen), C.byref(done)), "p3_layer_timeline_ns")
    return seen.value, done.value


def p3_layer_latency_ns(plan, layer):
    host, dev = _i64(), _i64()
    _check(load().p3_layer_latency_ns(_h(plan), int(layer), C.byref(host), C.byref(dev)), "p3_layer_latency_ns")
    return host.value, dev.value


def p3_drain_status(plan):
    a, w, ph, c = _i32(), _i32(), _i32(), _i32()
    _check(load().p3_drain_status(_h(plan), C.byref(a), C.byref(w), C.byref(ph), C.byref(c)), "p3_drain_status")
    return {"selector_status": a.value, "worker_status": w.value, "phase": ph.value, "claimed": c.value}


def p3_selector_timeline_ns(plan):
    a, c = _i64(), _i64()
    _check(load().p3_selector_timeline_ns(_h(plan), C.byref(a), C.byref(c)), "p3_selector_timeline_ns")
    return a.value, c.value


def p3_profile_enable(plan, on=True):
    _check(load().p3_profile_enable(_h(plan), 1 if on else 0), "p3_profile_enable")


def p3_profile_read(plan, each=0):
    """(total ms, launches), and with each=n also a float32 array of the first n launches' kernel ms."""
    ms, n = C.c_double(), _i32()
    if not each:
        _check(load().p3_profile_read(_h(plan), C.byref(ms), C.byref(n), None, 0), "p3_profile_read")
        return ms.value, n.value
    arr = np.zeros(int(each), dtype=np.float32)
    _check(load().p3_profile_read(_h(plan), C.byref(ms), C.byref(n), arr.ctypes.data_as(_P(C.c_float)), int(each)),
           "p3_profile_read")
    return ms.value, n.value, arr[:min(int(each), n.value)].copy()
