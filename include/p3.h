/*
 * p3.h -- C ABI of the MI355X parameter-server hot path of P3
 * (Priority-based Parameter Propagation, Jayarajan et al., SysML'19).
 *
 * The library plays the role of the paper's P3Server on one GPU: the gradient
 * of every layer is cut into slices no larger than a threshold (Sec. 4,
 * Sec. 4.2), a slice inherits the priority of its layer -- earlier in forward
 * order = more urgent (Sec. 4) -- and ready slices are aggregated over the W
 * workers' gradient copies and SGD-updated most-urgent-first (Sec. 4.2), with
 * the updated parameters published as soon as they are written (Sec. 4.2: the
 * server sends a slice out right after updating it).  The W workers are W
 * gradient arenas resident in this GPU's memory.
 *
 * Conventions
 *  - Every function returns a status (0 = P3_OK, negative = error) unless noted;
 *    nothing throws, aborts or prints.
 *  - "host" pointers are ordinary CPU memory owned by the caller and only read
 *    or written during the call.  "device" pointers are GPU global memory owned
 *    by the caller; the library never frees or reallocates them and they must
 *    stay valid until the plan is destroyed or re-bound.
 *  - One plan is driven from one host thread, except p3_mark_ready, p3_abort
 *    and p3_wait_layer, which may be called from another thread while a live
 *    drain is running.
 *  - Layers are parameter tensors in forward order; layer 0 is the first the
 *    next forward pass needs.
 *
 * Arena layout.  Each worker's gradients, the weights and the momentum are
 * flat arrays of p3_arena_elems() elements; layer l occupies
 * [p3_layer_offset(l), p3_layer_offset(l) + n_l).  Offsets are multiples of 64
 * elements; padding elements are never read or written.
 */
#ifndef P3_H_
#define P3_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct p3_plan_s p3_plan_t; /* opaque, created by p3_plan, freed by p3_destroy */

enum {
    P3_OK = 0,
    P3_ERR_ARG = -1,        /* null pointer, non-positive size, unknown enum value, misaligned arena */
    P3_ERR_STATE = -2,      /* call made in the wrong phase (e.g. drain before bind) */
    P3_ERR_RANGE = -3,      /* index or size out of range */
    P3_ERR_ALREADY = -4,    /* layer already marked ready in this iteration */
    P3_ERR_NOMEM = -5,      /* host or device allocation failed */
    P3_ERR_DEVICE = -6,     /* a HIP call failed, or no GPU / HIP runtime */
    P3_ERR_TIMEOUT = -7,    /* wait expired; a live drain was told to stop */
    P3_ERR_INCOMPLETE = -8  /* live drain ended with layers that were never marked */
};

enum { P3_GRAD_FP32 = 0, P3_GRAD_BF16 = 1 };
enum { P3_MODE_SNAPSHOT = 0, P3_MODE_LIVE = 1, P3_MODE_TICKED = 2 };
enum { P3_POLICY_PRIORITY = 0, P3_POLICY_FIFO = 1 };

#define P3_MAX_WORKERS 64

/* ---- planning: slicing and priorities (Sec. 4, Sec. 4.2; slice size Sec. 5.7) ----
 * layer_sizes: host array of n_layers element counts, forward order, each >= 1.
 * slice_elems: the maximum slice size (>= 1).  Layer l is cut into
 * ceil(n_l / slice_elems) slices: full ones and one shorter remainder.  Slices
 * get global ids g = 0..K-1 ordered by (layer, offset); ascending g is
 * descending urgency, so "highest priority first" is "smallest g first".
 * Host-only: touches no GPU.  *out receives the plan.
 * Errors: ARG (null, n_layers < 1, a size < 1, slice_elems < 1), RANGE (more
 * than 2^31-1 slices or a slice longer than 2^31-1 elements), NOMEM. */
int p3_plan(const int64_t* layer_sizes, int32_t n_layers, int64_t slice_elems, p3_plan_t** out);

/* One server's share (Sec. 4.1: with several servers the parameters are sharded
 * between them; Sec. 4.2: slices are handed to the servers round robin, which
 * spreads even a single heavy layer over all of them).  The plan owns the
 * slices whose global id is `shard` modulo n_shards and nothing else: marks,
 * drains, done flags and counts refer to the owned part of each layer.  The
 * arena layout (p3_layer_offset, p3_arena_elems) is that of the whole model,
 * so n_shards plans -- on n_shards devices, or one after another on one --
 * together update every parameter exactly once.  Owned slices are numbered
 * 0..p3_num_slices-1 in priority order; p3_slice_info takes these numbers,
 * p3_slice_global_id translates, p3_query_order reports global ids.  A layer
 * of which the shard owns nothing is done the moment it is marked.  Neighbouring
 * owned slices are not neighbours in memory, so every slice is a run of its own.
 * TICKED mode counts the shard's own claims.  p3_plan is the case (1, 0).
 * Errors: as p3_plan; ARG (n_shards < 1, shard outside 0..n_shards-1); RANGE
 * (the shard would own no slice). */
int p3_plan_sharded(const int64_t* layer_sizes, int32_t n_layers, int64_t slice_elems, int32_t n_shards,
                    int32_t shard, p3_plan_t** out);
/* Any pointer may be NULL.  global_slices: slices of the whole model. */
int p3_shard_info(const p3_plan_t* plan, int32_t* n_shards, int32_t* shard, int32_t* global_slices);
/* Global id of owned slice g, or a negative status (ARG, RANGE). */
int32_t p3_slice_global_id(const p3_plan_t* plan, int32_t g);

/* Frees the plan and every device/pinned buffer the library allocated for it.
 * Waits for an unfinished drain first (a live drain is told to stop), and, if
 * marks or waits were ever put on streams, for the device to finish them.  NULL ok. */
void p3_destroy(p3_plan_t* plan);

/* Introspection; host-only, valid right after p3_plan. Counts return -1 on NULL. */
int32_t p3_num_layers(const p3_plan_t* plan);
int32_t p3_num_slices(const p3_plan_t* plan);            /* K */
int64_t p3_num_elems(const p3_plan_t* plan);             /* N = sum n_l (of the owned slices, if sharded) */
int64_t p3_arena_elems(const p3_plan_t* plan);           /* >= N, includes alignment padding */
int64_t p3_layer_offset(const p3_plan_t* plan, int32_t layer);      /* element offset in an arena; -1 if bad */
int32_t p3_layer_first_slice(const p3_plan_t* plan, int32_t layer); /* -1 if bad */
int32_t p3_layer_num_slices(const p3_plan_t* plan, int32_t layer);  /* -1 if bad */
/* slice g -> parent layer (= priority), element offset inside the layer, length. RANGE if bad g. */
int p3_slice_info(const p3_plan_t* plan, int32_t g, int32_t* layer, int64_t* offset, int32_t* len);

/* ---- binding the data (the server's state: Sec. 4.1, KVServer keeps parameters) ----
 * grads: host array of W device pointers; grads[k] is worker k's gradient arena
 * (P3_GRAD_FP32: float, P3_GRAD_BF16: bfloat16 bit patterns), p3_arena_elems()
 * elements.  weights, momentum: device float arenas of the same length, updated
 * in place.  All arena pointers must be 16-byte aligned.  1 <= W <= P3_MAX_WORKERS.
 * Allocates the library's own control buffers on the current HIP device
 * (slice table, ready bitmap, work queue, order log; a few bytes per slice).
 * May be called again to re-bind other buffers when no drain is in flight.
 * Placement matters to the rate (several per cent): see p3_suggest_arena_stride.
 * Errors: ARG, RANGE (W), STATE (drain in flight), NOMEM, DEVICE. */
int p3_bind(p3_plan_t* plan, int32_t W, const void* const* grads, int32_t grad_dtype,
            float* weights, float* momentum);

/* Where to put the arenas.  Returns the distance in bytes to leave between the
 * bases of the W + 2 arenas (gradient copies, weights, momentum) when they are
 * carved from ONE device allocation -- the placement that was measured fastest
 * on MI355X: 2^29 gradient elements (2 GiB for fp32 copies, 1 GiB for bf16), or
 * the next multiple of that for longer arenas; arenas back to back were 2 to 5 %
 * slower, separate allocations slower still.  A hint only: any 16-byte aligned
 * placement is accepted by p3_bind.  Host-only.  Negative: ARG. */
int64_t p3_suggest_arena_stride(const p3_plan_t* plan, int32_t grad_dtype);

/* SGD hyper-parameters, taken by the next drain.  Per element, in fp32 with one
 * rounding per operation and no fused multiply-add:
 *   s = g_0 + g_1 + ... + g_{W-1}   (left to right; bf16 widened exactly)
 *   if rescale != 1: s = rescale*s ;  if wd != 0: s = s + wd*w
 *   m' = mu*m - lr*s ;  w' = w + m'
 * (The server's work on a key once all workers have pushed it: Sec. 2, Sec. 4.1.)
 * Defaults: lr 0.1, mu 0.9, rescale 1, wd 0. */
int p3_set_hyper(p3_plan_t* plan, float lr, float mu, float rescale, float wd);

/* How p3_drain decides what is ready (Sec. 4.2: producer/consumer through a
 * priority queue).  In every mode a claim takes the ready, unclaimed slice of
 * smallest g and is never revoked (the consumer finishes the slice it took).
 *  SNAPSHOT  a drain claims exactly the slices of layers marked before the call.
 *  LIVE      one drain per iteration runs while the host keeps marking layers;
 *            it ends when all K slices are claimed, on p3_abort, or when its
 *            watchdog expires.
 *  TICKED    layers marked before the call become ready at logical tick
 *            release_tick[l] (host array, n_layers entries, >= 0); the tick
 *            counter advances by one per claim and jumps over idle gaps.
 *            Deterministic model of backward propagation releasing layers
 *            while earlier ones are still being served (Sec. 1.1 preemption).
 * Takes effect at the next p3_begin_iter.  Errors: ARG (bad mode, null or
 * negative ticks). */
int p3_set_mode(p3_plan_t* plan, int32_t mode, const int64_t* release_tick);

/* Which ready slice the selector claims next.
 *  PRIORITY  (default) the paper's rule: the most urgent ready slice, i.e. the
 *            smallest global slice id (Sec. 4: priority = position of the layer
 *            in forward order; Sec. 4.2: the highest-priority slice goes first).
 *  FIFO      the baseline the paper argues against (Sec. 3, "aggressive"
 *            synchronisation): layers are served whole in the order they
 *            became ready -- the order of the marks in SNAPSHOT and LIVE mode,
 *            ascending release tick in TICKED mode (among equal ticks the later
 *            layer first, as backward produces them).  Slicing does not change
 *            this order; it is kept as the comparison arm for the layer-0
 *            latency argument.
 * Same arithmetic, same kernel; only the claim order differs.  Takes effect at
 * the next p3_begin_iter.  Errors: ARG. */
int p3_set_policy(p3_plan_t* plan, int32_t policy);

/* Launch shape and look-ahead.  Pass 0 to keep a value.
 *  tile_elems      work unit handed to one workgroup (multiple of 256, <= 2^20);
 *                  default: one step of a workgroup, 3328 elements
 *  wgs_per_cu      resident workgroups per compute unit the drain kernel uses
 *  lookahead_tiles LIVE only: how far the selector may run ahead of the workers
 *                  while layers are still unmarked; bounds how long a newly
 *                  ready urgent layer waits behind already claimed work
 *                  (default: two tiles per workgroup; once every layer of the
 *                  iteration is marked nothing can overtake any more and the
 *                  selector claims without this limit)
 *  watchdog_ms     no wait inside the kernel (for marks, for the selector) lasts
 *                  longer than this; default 10000
 * tile_elems and wgs_per_cu take effect at the next p3_begin_iter, the other
 * two at the next p3_drain.  Errors: ARG. */
int p3_set_tuning(p3_plan_t* plan, int32_t tile_elems, int32_t wgs_per_cu,
                  int32_t lookahead_tiles, int32_t watchdog_ms);

/* Leave n_cus compute units to other streams.  A drain launch normally puts a
 * workgroup on every compute unit and holds them until the iteration is
 * applied; a LIVE drain, or one that waits for marks made on a producer stream
 * (p3_mark_ready_on_stream), would then keep the producer's own kernels (the
 * backward pass that the transfer is meant to overlap: Sec. 3, Sec. 4.2)
 * from being scheduled until its wait runs out.  With n_cus > 0 the launch has
 * that many fewer workgroups, so the producer always finds free units; the
 * aggregation rate drops in proportion.  0 (default) uses the whole device; at
 * least two workgroups are always launched.
 * Takes effect at the next p3_begin_iter.  Errors: ARG. */
int p3_set_reserved_cus(p3_plan_t* plan, int32_t n_cus);

/* How a drain is put on the stream.  1 (default): one persistent launch in
 * which workgroup 0 selects while the others already work (what LIVE always
 * uses); a workgroup owns its compute unit.  0: two launches for a SNAPSHOT or
 * TICKED drain, the selector (one workgroup) and then the workers over the
 * finished work queue; no workgroup waits for another.  2: the persistent
 * launch with workgroups of 256 lanes and a quarter of the register file, which
 * leave room on every compute unit for workgroups of other kernels: a live
 * drain launched before a backward pass on another stream then runs beside it
 * instead of in front of it (Sec. 4: synchronisation overlapped with the
 * backward pass).  Alone it streams at two thirds of the default's rate; a
 * kernel whose wavefronts take a SIMD's whole register file still cannot start
 * beside it (p3_set_reserved_cus is for those).  Results are the same bits in
 * all three.  0 and 1 are taken by the next p3_drain, a change to or from 2 by
 * the next p3_begin_iter (the default tile size differs).  Errors: ARG. */
#define P3_LAUNCH_SPLIT 0
#define P3_LAUNCH_FUSED 1
#define P3_LAUNCH_LEAN 2
int p3_set_launch(p3_plan_t* plan, int32_t persistent);

/* ---- one iteration ----
 * p3_begin_iter: forget ready/claimed/done state and the order log; apply a
 *   pending mode or tuning change (which first waits for queued drains).
 *   STATE if not bound, or a LIVE drain is still running; NOMEM/DEVICE if the
 *   work queue cannot be allocated. */
int p3_begin_iter(p3_plan_t* plan);

/* All W gradient copies of `layer` are complete: all its slices enter the ready
 * set at once (Sec. 4.1: the server acts on a key once every worker has pushed
 * it; Sec. 4.2: the producer enqueues all slices of a layer together).
 * Host store only -- no kernel launch, no stream work.
 * Errors: STATE (no iteration begun), RANGE (bad layer), ALREADY (marked twice). */
int p3_mark_ready(p3_plan_t* plan, int32_t layer);

/* The same for n layers at once, in the order of the (host) array: what n calls
 * of p3_mark_ready would do, for callers whose call overhead is comparable to
 * the drain itself (a model of many small tensors driven from a scripting
 * language).  Stops at the first layer that fails and returns its error; the
 * layers before it stay marked.  n = 0 is allowed.
 * Errors: ARG (null array, n < 0), then as p3_mark_ready. */
int p3_mark_ready_many(p3_plan_t* plan, const int32_t* layers, int32_t n);

/* p3_mark_ready as the next operation of a HIP stream (a hipStream_t; NULL = the
 * default stream): the layer becomes ready when the stream has executed
 * everything enqueued before this call -- typically the kernels that produce the
 * layer's gradients (Sec. 4.2: the producer side hands a layer over when its
 * gradients are complete) -- without the host waiting for them.  The layer's
 * place in mark order is taken now (so ALREADY, RANGE and STATE are reported
 * now), and marks are taken by the selector in mark order: a mark that its
 * stream has not reached yet holds back the marks made after it.  A SNAPSHOT or
 * TICKED drain issued after this call waits on the device, within its time
 * limit, for the mark to arrive; it need not be ordered behind the producer
 * stream by the caller (if the mark does not arrive in that time the drain ends
 * with nothing more claimed and p3_sync reports INCOMPLETE).  The gradients must
 * be written by operations that precede the mark on that stream.  A drain that
 * occupies every compute unit while it waits keeps the producer's kernels from
 * starting: see p3_set_reserved_cus and p3_set_launch(plan, P3_LAUNCH_LEAN).
 * The same holds, whatever the launch, when the drain's stream and the
 * producer's share a hardware queue: HIP serves its streams through a few of
 * them (four by default), two streams on one queue run one after the other,
 * and which streams share one is not documented -- check that a kernel of one
 * stream starts while a kernel of the other is running before relying on it
 * (a drain that waits in vain ends by its time limit).  host_ns of
 * p3_layer_latency_ns counts from this call, not from the moment the stream
 * reaches the mark.
 * Errors: as p3_mark_ready, DEVICE. */
int p3_mark_ready_on_stream(p3_plan_t* plan, int32_t layer, void* producer_stream);

/* The consumer's counterpart: everything enqueued on consumer_stream (a
 * hipStream_t) after this call runs only once `layer` has been updated in this
 * iteration and its new weights are visible to the device -- the next forward
 * pass can be enqueued layer by layer behind such waits without the host
 * watching the flags (Sec. 3: the forward step of a layer needs that layer's
 * parameters back, nothing else; Sec. 4: that is why the first layers go first).
 * The wait is a one-lane kernel that polls the layer's done flag; it ends after
 * timeout_ms at the latest (negative: the plan's watchdog), and then what
 * follows it runs on whatever the weights hold: p3_stream_wait_expired tells.
 * Call it after p3_begin_iter of the iteration it refers to.  A drain that
 * covers every compute unit leaves no room for the consumer's kernels until it
 * ends: see p3_set_reserved_cus.  HIP maps streams onto a few hardware queues
 * (four by default); a stream that shares its queue with the waiting one may be
 * held up behind the wait, so keep the streams in use (drain, producer,
 * consumer) within that number.  Errors: STATE, RANGE, DEVICE. */
int p3_wait_layer_on_stream(p3_plan_t* plan, int32_t layer, void* consumer_stream, int32_t timeout_ms);
/* 1 if a p3_wait_layer_on_stream of the current iteration has run out of time
 * (as far as the consumer stream has got: synchronise it first), else 0;
 * negative: ARG, STATE. */
int p3_stream_wait_expired(p3_plan_t* plan);

/* Aggregate + update ready slices in priority order (Sec. 4.2).  Asynchronous:
 * enqueues one persistent kernel on `hip_stream` (a hipStream_t; NULL = default
 * stream) and returns.  Selection, tile hand-out, arithmetic and completion
 * flags all run on the device with no host round trip per slice.
 * Errors: STATE (not bound / no iteration begun / LIVE drain already issued),
 * DEVICE. A SNAPSHOT or TICKED drain with nothing newly marked is P3_OK and
 * launches nothing. */
int p3_drain(p3_plan_t* plan, void* hip_stream);

/* Wait until every drain issued so far has finished.  timeout_ms < 0: no limit.
 * On expiry the running drain is told to stop (it finishes the tiles already
 * handed out), is waited for, and TIMEOUT is returned.  INCOMPLETE if a drain
 * ended early (abort, watchdog) or a LIVE drain ended before all K slices were
 * claimed.  DEVICE on a HIP error. */
int p3_sync(p3_plan_t* plan, int32_t timeout_ms);

/* Non-blocking: P3_OK if every drain issued so far has finished, TIMEOUT if one
 * is still running (nothing is stopped), DEVICE on a HIP error. */
int p3_poll(p3_plan_t* plan);

/* Ask a running LIVE drain to stop claiming; already claimed slices finish. */
int p3_abort(p3_plan_t* plan);

/* Block until `layer` is fully updated in this iteration and its weights are
 * visible to later work on the GPU (Sec. 4.2: an updated slice is sent out at
 * once; the next forward pass needs layer 0 first, Sec. 3).  Polls a flag the
 * kernel writes to pinned host memory.  TIMEOUT on expiry (timeout_ms < 0: none). */
int p3_wait_layer(p3_plan_t* plan, int32_t layer, int32_t timeout_ms);

/* ---- results for checking ----
 * p3_query_order: global slice ids in the order they were claimed in this
 * iteration, into host array out[cap]; waits for issued drains; returns the
 * count (<= K) or a negative status. */
int32_t p3_query_order(p3_plan_t* plan, int32_t* out, int32_t cap);
/* For each claim, how many p3_mark_ready calls of this iteration the selector
 * had observed when it made the claim (non-decreasing).  Same return rule. */
int32_t p3_query_trace(p3_plan_t* plan, int32_t* epoch_seen, int32_t cap);
/* Layer latency of this iteration: host_ns from entry of p3_mark_ready(layer)
 * to the host seeing the layer's done flag (needs p3_wait_layer or p3_sync to
 * have observed it); dev_ns from the selector first seeing the layer ready to
 * its last tile retiring, by the GPU's constant-rate clock.  Either pointer
 * may be NULL.  STATE if the layer has not completed. */
int p3_layer_latency_ns(p3_plan_t* plan, int32_t layer, int64_t* host_ns, int64_t* dev_ns);
/* The same two device stamps of a completed layer on the time axis of the most
 * recent drain: nanoseconds from the selector's first instruction in that
 * launch to the selector seeing the layer ready (seen_ns) and to the layer
 * being visible (done_ns).  This is the "when does layer l come back" curve of
 * Sec. 3 (Fig. "Parameter synchronization").  A stamp taken by an earlier drain
 * of the iteration comes out negative.  Waits for issued drains.  Either
 * pointer may be NULL.  Errors: ARG, RANGE, STATE (layer not completed). */
int p3_layer_timeline_ns(p3_plan_t* plan, int32_t layer, int64_t* seen_ns, int64_t* done_ns);

/* Diagnostics of the most recent drain, read from the kernel's host mailbox
 * without waiting: how the selector ended (0 ok, 1 watchdog, 2 aborted,
 * 3 internal overflow), whether a worker gave up waiting (0 no, 1 yes), the
 * selector's progress code (1 entered .. 6 finished) and the number of slices
 * claimed so far in the iteration.  Any pointer may be NULL. */
int p3_drain_status(p3_plan_t* plan, int32_t* selector_status, int32_t* worker_status,
                    int32_t* phase, int32_t* claimed);

/* Selector timeline of the most recent drain, by the GPU's constant-rate clock:
 * nanoseconds from the selector's first instruction to the first growth of the
 * work queue (when the workers can start; -1 if it never grew) and to the end
 * of selection.  Waits for issued drains.  Either pointer may be NULL. */
int p3_selector_timeline_ns(p3_plan_t* plan, int64_t* first_publish_ns, int64_t* finished_ns);

/* Optional HIP-event bracketing of every drain kernel, on the drain's stream.
 * p3_profile_read: accumulated kernel milliseconds and launch count since the
 * last p3_profile_enable(plan, 1), and, into the host array each_ms[cap] (may be
 * NULL with cap 0), the kernel milliseconds of the first min(cap, launches)
 * launches one by one; waits for issued drains.  Errors: ARG, STATE, NOMEM. */
int p3_profile_enable(p3_plan_t* plan, int32_t on);
int p3_profile_read(p3_plan_t* plan, double* total_ms, int32_t* launches, float* each_ms, int32_t cap);

/* ---- one iteration that allocates nothing ----
 * For callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  What p3_bind + p3_begin_iter +
 * p3_mark_ready_many(ready_layers) + one SNAPSHOT p3_drain do, as one call that
 * makes no hipMalloc / hipFree and needs no bound plan: the library's control
 * data (slice and layer tables, ready bitmap, work queue, counters, completion
 * flags) lives in one static device array of about 310 KB per GPU, which limits
 * the plan to P3_STATIC_MAX_LAYERS layers and P3_STATIC_MAX_SLICES slices
 * (RANGE beyond that).  Only kernels are enqueued on hip_stream (no memset, no
 * copy); the call returns without waiting.
 *  plan          from p3_plan (not sharded); only read; need not be bound
 *  grads         host array of W device pointers, as in p3_bind
 *  weights, momentum   device arenas, updated in place
 *  ready_layers  host array of n_ready distinct layers, in mark order; their
 *                slices are claimed in priority order and processed
 *  order_out     device array of p3_num_slices(plan) int32: the claim order
 *  result_out    device array of 4 int32: slices claimed, selector status
 *                (0 ok), worker status (0 ok), layers whose update is complete
 * All calls on one GPU share that GPU's array, which keeps the previous call's
 * contents (the call clears what must start at zero): calls that overlap on one
 * GPU -- on different streams, or from different threads -- race; order them.
 * Errors: ARG (null, unknown dtype, misaligned arena, sharded plan), RANGE (W,
 * a layer index, plan beyond the static limits), ALREADY (a layer twice), DEVICE. */
#define P3_STATIC_MAX_LAYERS 256
#define P3_STATIC_MAX_SLICES 4096
int p3_drain_static(const p3_plan_t* plan, int32_t W, const void* const* grads, int32_t grad_dtype,
                    float* weights, float* momentum, float lr, float mu, float rescale, float wd,
                    const int32_t* ready_layers, int32_t n_ready, int32_t* order_out,
                    int32_t* result_out, void* hip_stream);

/* After a P3_ERR_DEVICE: the hipError_t value of the most recent failing HIP
 * call made by the library in this process (0 if none) and, if source_line is
 * not NULL, the line of the runtime source that made it.  Diagnostics only. */
int p3_last_hip_error(int* source_line);

/* Static description of a status code. Never NULL. */
const char* p3_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* P3_H_ */
