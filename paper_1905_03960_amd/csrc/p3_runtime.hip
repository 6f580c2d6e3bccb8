// Host side of the P3 hot-path library: the slice planner (integer only), the
// plan handle, argument checks, pinned host<->device mailboxes and the launch
// of the persistent drain kernel.  Public contract: include/p3.h.

#include <hip/hip_runtime.h>

#include <atomic>
#include <chrono>
#include <cstring>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "p3.h"
#include "p3_internal.h"
#include "p3_planner.h"

namespace {

constexpr int kEventRing = 4;            // iterations whose marks may coexist in the mark ring

inline int64_t now_ns() {
    return std::chrono::duration_cast<std::chrono::nanoseconds>(
               std::chrono::steady_clock::now().time_since_epoch())
        .count();
}

// Last failing HIP call of this process (code and source line), for p3_last_hip_error.
std::atomic<int> g_hip_code{0};
std::atomic<int> g_hip_line{0};
inline hipError_t note(hipError_t e, int line) {
    if (e != hipSuccess && e != hipErrorNotReady) {
        g_hip_code.store(static_cast<int>(e));
        g_hip_line.store(line);
    }
    return e;
}
#define HIPC(call) note((call), __LINE__)

struct ProfPair {
    hipEvent_t start = nullptr, stop = nullptr;
};

}  // namespace

struct p3_plan_s : P3PlanTables {
    // ---- plan (host only; filled by p3_plan): the inherited tables ----

    // ---- configuration ----
    float lr = 0.1f, mu = 0.9f, rescale = 1.0f, wd = 0.0f;
    int32_t mode = P3_MODE_SNAPSHOT;
    int32_t policy = P3_POLICY_PRIORITY, next_policy = P3_POLICY_PRIORITY;
    std::vector<int64_t> release;
    int32_t tile_elems = 0;            // 0: one step of the workgroup (P3_BLOCK lanes x 4 elements)
    int32_t wgs_per_cu = 1;
    int32_t reserved_cus = 0, next_reserved_cus = -1;   // compute units left to other streams
    int32_t lookahead = 0;             // 0: derive from the grid
    int32_t watchdog_ms = 10000;
    int32_t persistent = 1;            // SNAPSHOT/TICKED: one fused launch (1) or selector + workers (0)
    int32_t lean = 0, next_lean = -1;  // 1: the build with small workgroups that share their compute unit
    int32_t count_set = 0;             // which of the two sets of per-layer counts the current iteration uses
    // set by p3_set_mode / p3_set_tuning, applied by the next p3_begin_iter
    bool pending_mode = false, pending_tuning = false;
    int32_t next_mode = P3_MODE_SNAPSHOT;
    std::vector<int64_t> next_release;
    int32_t next_tile_elems = 0, next_wgs_per_cu = 0;

    // ---- binding ----
    bool bound = false;
    int device = -1;
    int32_t W = 0, dtype = 0;
    P3GradPtrs grads{};
    float* w = nullptr;
    float* m = nullptr;
    int num_cu = 0;
    int clock_khz = 100000;
    unsigned grid = 0;
    uint32_t run_cap = 0;
    int64_t tiles_total = 0;           // grid cells touched by the plan's slices at the current tile size

    // device buffers owned by the library
    P3SliceDev* d_slices = nullptr;
    P3LayerDev* d_layers = nullptr;
    int64_t* d_release = nullptr;
    unsigned long long* d_bitmap = nullptr;
    uint8_t* d_layer_state = nullptr;
    P3Run* d_runq = nullptr;
    int32_t* d_order = nullptr;
    int32_t* d_epoch = nullptr;
    unsigned long long* d_layer_done = nullptr;
    uint32_t* d_layer_req = nullptr;
    int32_t* d_fifo = nullptr;
    uint64_t* d_t_seen = nullptr;
    P3Ctl* d_ctl = nullptr;
    // pinned host buffers
    P3HostShared* hs = nullptr;
    unsigned long long* mark_log = nullptr;   // entry = (low 32 bits of absolute index + 1) << 32 | layer
    bool stream_ops = false;           // a mark or wait kernel was ever put on a caller's stream
    bool stream_marks = false;         // this iteration has marks that a stream will make (no marks with the launch then)
    uint32_t mark_cap = 0;
    uint32_t* done_flag = nullptr;
    uint32_t* wait_expired = nullptr;  // set to the iteration's number by a stream wait that ran out of time
    uint64_t* t_seen = nullptr;
    uint64_t* t_done = nullptr;

    // ---- iteration state (host) ----
    std::mutex mu_host;                // guards marks
    bool iter_open = false;
    uint32_t iter_seq = 0;
    uint64_t marks_total = 0;          // absolute
    uint64_t epoch_base = 0;
    uint64_t drained_upto = 0;         // marks covered by issued SNAPSHOT/TICKED drains
    std::vector<uint8_t> marked;
    std::vector<int64_t> t_mark_ns, t_seen_done_ns;
    bool first_drain = true;
    bool live_issued = false;
    bool in_flight = false;
    int last_slot = 0;                 // ev_iter[last_slot] was recorded behind the most recent drain
    hipEvent_t ev_iter[kEventRing] = {nullptr, nullptr, nullptr, nullptr};
    bool ev_iter_used[kEventRing] = {false, false, false, false};

    // ---- profiling ----
    bool prof_on = false;
    std::vector<ProfPair> prof_pool;
    size_t prof_used = 0;
    double prof_ms = 0.0;
    int32_t prof_launches = 0;
    std::vector<float> prof_each;      // kernel time of every bracketed launch since profiling was switched on
};

namespace {

// A mark log entry: valid for absolute position `index` when its upper half says so.
unsigned long long mark_entry(uint64_t index, int32_t layer) {
    return (static_cast<unsigned long long>(static_cast<uint32_t>(index + 1)) << 32) | static_cast<uint32_t>(layer);
}

int32_t tiles_of(int64_t len, int32_t tile) { return static_cast<int32_t>((len + tile - 1) / tile); }

int64_t total_tiles(const p3_plan_s* p, int32_t tile) { return p3_planner_total_tiles(*p, tile); }

void free_device(p3_plan_s* p) {
    if (p->device >= 0) (void)hipSetDevice(p->device);
    auto fd = [](auto*& ptr) {
        if (ptr) (void)hipFree(ptr);
        ptr = nullptr;
    };
    auto fh = [](auto*& ptr) {
        if (ptr) (void)hipHostFree(ptr);
        ptr = nullptr;
    };
    fd(p->d_slices);
    fd(p->d_layers);
    fd(p->d_release);
    fd(p->d_bitmap);
    fd(p->d_layer_state);
    fd(p->d_runq);
    fd(p->d_order);
    fd(p->d_epoch);
    fd(p->d_layer_done);
    fd(p->d_layer_req);
    fd(p->d_fifo);
    fd(p->d_t_seen);
    fd(p->d_ctl);
    fh(p->hs);
    fh(p->mark_log);
    fh(p->done_flag);
    fh(p->wait_expired);
    fh(p->t_seen);
    fh(p->t_done);
    for (int i = 0; i < kEventRing; ++i) {
        if (p->ev_iter[i]) (void)hipEventDestroy(p->ev_iter[i]);
        p->ev_iter[i] = nullptr;
        p->ev_iter_used[i] = false;
    }
    for (ProfPair& pp : p->prof_pool) {
        if (pp.start) (void)hipEventDestroy(pp.start);
        if (pp.stop) (void)hipEventDestroy(pp.stop);
    }
    p->prof_pool.clear();
    p->prof_used = 0;
    p->bound = false;
}

// Wait for everything issued.  A live drain that does not end within
// timeout_ms is told to stop and then waited for.
int wait_idle(p3_plan_s* p, int32_t timeout_ms, bool* timed_out) {
    if (timed_out) *timed_out = false;
    if (!p->in_flight) return P3_OK;
    const int64_t t0 = now_ns();
    for (;;) {
        hipError_t e = hipEventQuery(p->ev_iter[p->last_slot]);
        if (e == hipSuccess) break;
        if (e != hipErrorNotReady) return P3_ERR_DEVICE;
        if (timeout_ms >= 0 && now_ns() - t0 > static_cast<int64_t>(timeout_ms) * 1000000) {
            if (timed_out) *timed_out = true;
            std::atomic_thread_fence(std::memory_order_seq_cst);
            reinterpret_cast<std::atomic<uint32_t>*>(&p->hs->abort_flag)->store(1u, std::memory_order_release);
            if (HIPC(hipEventSynchronize(p->ev_iter[p->last_slot])) != hipSuccess) return P3_ERR_DEVICE;
            break;
        }
        std::this_thread::yield();
    }
    p->in_flight = false;
    return P3_OK;
}

void collect_profile(p3_plan_s* p) {
    for (size_t i = 0; i < p->prof_used; ++i) {
        float ms = 0.f;
        if (HIPC(hipEventElapsedTime(&ms, p->prof_pool[i].start, p->prof_pool[i].stop)) == hipSuccess) {
            p->prof_ms += ms;
            p->prof_launches += 1;
            p->prof_each.push_back(ms);
        }
    }
    p->prof_used = 0;
}

}  // namespace

extern "C" {

int p3_last_hip_error(int* source_line) {
    if (source_line) *source_line = g_hip_line.load();
    return g_hip_code.load();
}

const char* p3_strerror(int status) {
    switch (status) {
        case P3_OK: return "ok";
        case P3_ERR_ARG: return "invalid argument";
        case P3_ERR_STATE: return "call not valid in this state";
        case P3_ERR_RANGE: return "index or size out of range";
        case P3_ERR_ALREADY: return "layer already marked ready in this iteration";
        case P3_ERR_NOMEM: return "out of memory";
        case P3_ERR_DEVICE: return "HIP call failed or no GPU";
        case P3_ERR_TIMEOUT: return "timed out";
        case P3_ERR_INCOMPLETE: return "drain ended before every layer was marked ready";
        default: return "unknown status";
    }
}

// ------------------------------------------------------------------ planner ----
int p3_plan_sharded(const int64_t* layer_sizes, int32_t n_layers, int64_t slice_elems, int32_t n_shards,
                    int32_t shard, p3_plan_t** out) {
    if (!out) return P3_ERR_ARG;
    *out = nullptr;
    p3_plan_s* p = new (std::nothrow) p3_plan_s;
    if (!p) return P3_ERR_NOMEM;
    int rc = P3_ERR_NOMEM;
    try {
        rc = p3_planner_build(layer_sizes, n_layers, slice_elems, n_shards, shard, *p);
        if (rc == P3_OK) {
            p->marked.assign(static_cast<size_t>(n_layers), 0);
            p->t_mark_ns.assign(static_cast<size_t>(n_layers), 0);
            p->t_seen_done_ns.assign(static_cast<size_t>(n_layers), 0);
        }
    } catch (const std::bad_alloc&) {
        rc = P3_ERR_NOMEM;
    }
    if (rc != P3_OK) {
        delete p;
        return rc;
    }
    *out = p;
    return P3_OK;
}

int p3_plan(const int64_t* layer_sizes, int32_t n_layers, int64_t slice_elems, p3_plan_t** out) {
    return p3_plan_sharded(layer_sizes, n_layers, slice_elems, 1, 0, out);
}

int p3_shard_info(const p3_plan_t* p, int32_t* n_shards, int32_t* shard, int32_t* global_slices) {
    if (!p) return P3_ERR_ARG;
    if (n_shards) *n_shards = p->n_shards;
    if (shard) *shard = p->shard;
    if (global_slices) *global_slices = p->K_global;
    return P3_OK;
}

int32_t p3_slice_global_id(const p3_plan_t* p, int32_t g) {
    if (!p) return P3_ERR_ARG;
    if (g < 0 || g >= p->K) return P3_ERR_RANGE;
    return p->global_id[static_cast<size_t>(g)];
}

void p3_destroy(p3_plan_t* p) {
    if (!p) return;
    if (p->bound) {
        (void)hipSetDevice(p->device);
        if (p->in_flight) {
            bool to = false;
            (void)wait_idle(p, p->live_issued ? 0 : -1, &to);
        }
        // mark and wait kernels sit on streams of the caller's and point into the pinned buffers
        // freed below: let them finish (they are bounded) before the memory goes
        if (p->stream_ops) (void)hipDeviceSynchronize();
        free_device(p);
    }
    delete p;
}

int32_t p3_num_layers(const p3_plan_t* p) { return p ? p->L : -1; }
int32_t p3_num_slices(const p3_plan_t* p) { return p ? p->K : -1; }
int64_t p3_num_elems(const p3_plan_t* p) { return p ? p->N : -1; }
int64_t p3_arena_elems(const p3_plan_t* p) { return p ? p->arena : -1; }
int64_t p3_layer_offset(const p3_plan_t* p, int32_t l) {
    return (p && l >= 0 && l < p->L) ? p->offset[l] : -1;
}
int32_t p3_layer_first_slice(const p3_plan_t* p, int32_t l) {
    return (p && l >= 0 && l < p->L) ? p->layers[l].first : -1;
}
int32_t p3_layer_num_slices(const p3_plan_t* p, int32_t l) {
    return (p && l >= 0 && l < p->L) ? p->layers[l].count : -1;
}
int p3_slice_info(const p3_plan_t* p, int32_t g, int32_t* layer, int64_t* offset, int32_t* len) {
    if (!p) return P3_ERR_ARG;
    if (g < 0 || g >= p->K) return P3_ERR_RANGE;
    const P3SliceDev& s = p->slices[g];
    if (layer) *layer = s.layer;
    if (offset) *offset = s.start - p->offset[s.layer];
    if (len) *len = s.len;
    return P3_OK;
}

// ------------------------------------------------------------------ binding ----
// The grid cell the runs are cut on.  Unless tuned, one step of a workgroup: every lane four
// consecutive parameters (more steps per tile were measured to cost bandwidth).
static int32_t tile_of_plan(const p3_plan_s* p) {
    if (p->tile_elems) return p->tile_elems;
    return p->lean ? P3_TILE_LEAN : P3_BLOCK * 4;
}

static int alloc_queue(p3_plan_s* p) {
    const int64_t t = total_tiles(p, tile_of_plan(p));
    if (t > INT32_MAX - 65536) return P3_ERR_RANGE;
    p->tiles_total = t;
    // tiles are numbered with 32 bits; the queue itself has at most one run per slice
    if (!p->d_runq) {
        if (HIPC(hipMalloc(&p->d_runq, sizeof(P3Run) * static_cast<size_t>(p->K))) != hipSuccess) return P3_ERR_NOMEM;
        p->run_cap = static_cast<uint32_t>(p->K);
    }
    return P3_OK;
}

static int size_grid(p3_plan_s* p) {
    int occ = 0;
    if (HIPC(static_cast<hipError_t>((p->lean ? p3_drain_occupancy_lean : p3_drain_occupancy)(p->W, p->dtype, 1, &occ))) !=
            hipSuccess ||
        occ < 1)
        return P3_ERR_DEVICE;
    int per_cu = p->wgs_per_cu < occ ? p->wgs_per_cu : occ;   // never more than can be co-resident
    if (per_cu < 1) per_cu = 1;
    int cus = p->num_cu - p->reserved_cus;
    // at least two workgroups: in a live drain workgroup 0 selects for as long as marks are outstanding,
    // and somebody else has to work off what it publishes
    if (cus < 2) cus = p->num_cu < 2 ? 1 : 2;
    p->grid = static_cast<unsigned>(cus) * static_cast<unsigned>(per_cu);
    // a model of fewer tiles than that is not worth more workgroups than tiles: every workgroup
    // launched has to be dispatched, registered with its XCD and counted out again
    const int64_t tiles = p->tiles_total;
    if (tiles < static_cast<int64_t>(p->grid)) p->grid = tiles < 2 ? 2u : static_cast<unsigned>(tiles);
    return P3_OK;
}

int p3_bind(p3_plan_t* p, int32_t W, const void* const* grads, int32_t grad_dtype,
            float* weights, float* momentum) {
    if (!p || !grads || !weights || !momentum) return P3_ERR_ARG;
    if (grad_dtype != P3_GRAD_FP32 && grad_dtype != P3_GRAD_BF16) return P3_ERR_ARG;
    if (W < 1 || W > P3_MAX_WORKERS) return P3_ERR_RANGE;
    auto misaligned = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) != 0; };
    if (misaligned(weights) || misaligned(momentum)) return P3_ERR_ARG;
    for (int32_t k = 0; k < W; ++k)
        if (!grads[k] || misaligned(grads[k])) return P3_ERR_ARG;
    if (p->in_flight) {
        if (p->live_issued) return P3_ERR_STATE;
        if (int rc = wait_idle(p, -1, nullptr)) return rc;
    }

    if (!p->bound) {
        int dev = 0;
        if (HIPC(hipGetDevice(&dev)) != hipSuccess) return P3_ERR_DEVICE;
        hipDeviceProp_t prop;
        if (HIPC(hipGetDeviceProperties(&prop, dev)) != hipSuccess) return P3_ERR_DEVICE;
        p->device = dev;
        p->num_cu = prop.multiProcessorCount;
        int khz = 0;
        if (HIPC(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev)) == hipSuccess && khz > 0)
            p->clock_khz = khz;

        const size_t K = static_cast<size_t>(p->K), L = static_cast<size_t>(p->L);
        const size_t n_words = (K + 63) / 64;
        p->mark_cap = static_cast<uint32_t>(kEventRing * L < 64 ? 64 : kEventRing * L);
        bool ok = true;
        auto dm = [&ok](auto** ptr, size_t bytes) {
            if (ok && HIPC(hipMalloc(reinterpret_cast<void**>(ptr), bytes)) != hipSuccess) ok = false;
        };
        // mailboxes a running kernel and the host both touch: coherent (fine-grained) pinned memory
        auto hm = [&ok](auto** ptr, size_t bytes) {
            if (ok && HIPC(hipHostMalloc(reinterpret_cast<void**>(ptr), bytes, hipHostMallocCoherent)) != hipSuccess)
                ok = false;
        };
        dm(&p->d_slices, sizeof(P3SliceDev) * K);
        dm(&p->d_layers, sizeof(P3LayerDev) * L);
        dm(&p->d_release, sizeof(int64_t) * L);
        dm(&p->d_bitmap, sizeof(unsigned long long) * n_words);
        dm(&p->d_layer_state, L);
        dm(&p->d_order, sizeof(int32_t) * K);
        dm(&p->d_epoch, sizeof(int32_t) * K);
        dm(&p->d_layer_done, sizeof(unsigned long long) * L * 2);     // two sets: iterations alternate (P3DrainArgs)
        dm(&p->d_layer_req, sizeof(uint32_t) * L * 2);
        dm(&p->d_fifo, sizeof(int32_t) * L);
        dm(&p->d_t_seen, sizeof(uint64_t) * L);
        dm(&p->d_ctl, sizeof(P3Ctl));
        hm(&p->hs, sizeof(P3HostShared));
        hm(&p->mark_log, sizeof(unsigned long long) * p->mark_cap);
        hm(&p->done_flag, sizeof(uint32_t) * L);
        hm(&p->wait_expired, sizeof(uint32_t));
        hm(&p->t_seen, sizeof(uint64_t) * L);
        hm(&p->t_done, sizeof(uint64_t) * L);
        for (int i = 0; ok && i < kEventRing; ++i)
            if (HIPC(hipEventCreateWithFlags(&p->ev_iter[i], hipEventDisableTiming)) != hipSuccess) ok = false;
        if (!ok) {
            free_device(p);
            return P3_ERR_NOMEM;
        }
        std::memset(p->hs, 0, sizeof(P3HostShared));
        std::memset(p->mark_log, 0, sizeof(unsigned long long) * p->mark_cap);
        std::memset(p->done_flag, 0, sizeof(uint32_t) * L);
        *p->wait_expired = 0u;
        std::memset(p->t_seen, 0, sizeof(uint64_t) * L);
        std::memset(p->t_done, 0, sizeof(uint64_t) * L);
        P3Ctl ctl;
        std::memset(&ctl, 0, sizeof ctl);
        ctl.final_runs = P3_NONE;
        ctl.lo_word = static_cast<uint32_t>(n_words);
        std::vector<int64_t> rel(L, 0);
        if (!p->release.empty()) rel = p->release;
        hipError_t e = HIPC(hipMemcpy(p->d_slices, p->slices.data(), sizeof(P3SliceDev) * K, hipMemcpyHostToDevice));
        if (e == hipSuccess) e = HIPC(hipMemcpy(p->d_layers, p->layers.data(), sizeof(P3LayerDev) * L, hipMemcpyHostToDevice));
        if (e == hipSuccess) e = HIPC(hipMemcpy(p->d_release, rel.data(), sizeof(int64_t) * L, hipMemcpyHostToDevice));
        if (e == hipSuccess) e = HIPC(hipMemcpy(p->d_ctl, &ctl, sizeof ctl, hipMemcpyHostToDevice));
        if (e == hipSuccess) e = HIPC(hipMemset(p->d_bitmap, 0, sizeof(unsigned long long) * n_words));
        if (e == hipSuccess) e = HIPC(hipMemset(p->d_layer_state, 0, L));
        if (e == hipSuccess) e = HIPC(hipMemset(p->d_layer_done, 0, sizeof(unsigned long long) * L * 2));
        if (e == hipSuccess) e = HIPC(hipMemset(p->d_layer_req, 0, sizeof(uint32_t) * L * 2));
        if (e == hipSuccess) e = HIPC(hipMemset(p->d_order, 0xff, sizeof(int32_t) * K));
        if (e == hipSuccess) e = HIPC(hipMemset(p->d_epoch, 0, sizeof(int32_t) * K));
        if (e == hipSuccess) e = HIPC(hipDeviceSynchronize());
        if (e != hipSuccess) {
            free_device(p);
            return P3_ERR_DEVICE;
        }
        p->W = W;                 // needed by alloc/size below
        p->dtype = grad_dtype;
        if (int rc = alloc_queue(p)) {
            free_device(p);
            return rc;
        }
        p->bound = true;
    } else {
        if (HIPC(hipSetDevice(p->device)) != hipSuccess) return P3_ERR_DEVICE;
    }
    p->W = W;
    p->dtype = grad_dtype;
    std::memset(&p->grads, 0, sizeof p->grads);
    for (int32_t k = 0; k < W; ++k) p->grads.p[k] = grads[k];
    p->w = weights;
    p->m = momentum;
    if (int rc = size_grid(p)) return rc;
    return P3_OK;
}

// Measured on MI355X (one allocation, all arenas `stride` apart, the VGG-19-, seq2seq- and ResNet-50-shaped
// drains): 2^29 elements of the gradient type between the arenas' bases -- 2 GiB with fp32 copies, 1 GiB
// with bf16 copies -- was the best or within 0.5 % of the best of eight spacings tried, the arenas back to
// back 2 to 5 % slower.  An arena longer than that gets the next multiple.
int64_t p3_suggest_arena_stride(const p3_plan_t* p, int32_t grad_dtype) {
    if (!p) return P3_ERR_ARG;
    if (grad_dtype != P3_GRAD_FP32 && grad_dtype != P3_GRAD_BF16) return P3_ERR_ARG;
    const int64_t unit = (static_cast<int64_t>(1) << 29) * (grad_dtype == P3_GRAD_BF16 ? 2 : 4);
    const int64_t bytes = p->arena * 4;                     // weights and momentum are fp32 whatever the gradients are
    return (bytes + unit - 1) / unit * unit;
}

int p3_set_hyper(p3_plan_t* p, float lr, float mu, float rescale, float wd) {
    if (!p) return P3_ERR_ARG;
    p->lr = lr;
    p->mu = mu;
    p->rescale = rescale;
    p->wd = wd;
    return P3_OK;
}

int p3_set_mode(p3_plan_t* p, int32_t mode, const int64_t* release_tick) {
    if (!p) return P3_ERR_ARG;
    if (mode != P3_MODE_SNAPSHOT && mode != P3_MODE_LIVE && mode != P3_MODE_TICKED) return P3_ERR_ARG;
    if (mode == P3_MODE_TICKED) {
        if (!release_tick) return P3_ERR_ARG;
        for (int32_t l = 0; l < p->L; ++l)
            if (release_tick[l] < 0) return P3_ERR_ARG;
        p->next_release.assign(release_tick, release_tick + p->L);
    }
    p->next_mode = mode;
    p->pending_mode = true;
    return P3_OK;
}

int p3_set_policy(p3_plan_t* p, int32_t policy) {
    if (!p) return P3_ERR_ARG;
    if (policy != P3_POLICY_PRIORITY && policy != P3_POLICY_FIFO) return P3_ERR_ARG;
    p->next_policy = policy;
    p->pending_mode = true;
    return P3_OK;
}

int p3_set_tuning(p3_plan_t* p, int32_t tile_elems, int32_t wgs_per_cu, int32_t lookahead_tiles,
                  int32_t watchdog_ms) {
    if (!p) return P3_ERR_ARG;
    if (tile_elems < 0 || wgs_per_cu < 0 || lookahead_tiles < 0 || watchdog_ms < 0) return P3_ERR_ARG;
    if (tile_elems != 0 && (tile_elems % 256 != 0 || tile_elems > (1 << 20))) return P3_ERR_ARG;
    if (wgs_per_cu > 16) return P3_ERR_ARG;
    if (tile_elems) p->next_tile_elems = tile_elems;
    if (wgs_per_cu) p->next_wgs_per_cu = wgs_per_cu;
    if (tile_elems || wgs_per_cu) p->pending_tuning = true;
    if (lookahead_tiles) p->lookahead = lookahead_tiles;     // plain launch arguments: next drain
    if (watchdog_ms) p->watchdog_ms = watchdog_ms;
    return P3_OK;
}

int p3_set_reserved_cus(p3_plan_t* p, int32_t n_cus) {
    if (!p) return P3_ERR_ARG;
    if (n_cus < 0 || n_cus > 4096) return P3_ERR_ARG;
    p->next_reserved_cus = n_cus;
    p->pending_tuning = true;
    return P3_OK;
}

int p3_set_launch(p3_plan_t* p, int32_t persistent) {
    if (!p) return P3_ERR_ARG;
    if (persistent < 0 || persistent > 2) return P3_ERR_ARG;
    p->persistent = persistent != 0 ? 1 : 0;
    // the lean build has its own tile size and grid: like them, it changes at an iteration boundary
    p->next_lean = persistent == 2 ? 1 : 0;
    p->pending_tuning = true;
    return P3_OK;
}

// Mode, release ticks, tile size and grid change only at an iteration boundary:
// the device bookkeeping of an iteration (tiles per slice, release table) must
// not move under a drain that is already queued.
static int apply_pending(p3_plan_s* p) {
    if (!p->pending_mode && !p->pending_tuning) return P3_OK;
    if (int rc = wait_idle(p, -1, nullptr)) return rc;
    if (p->pending_mode) {
        if (p->next_mode == P3_MODE_TICKED) {
            if (HIPC(hipMemcpy(p->d_release, p->next_release.data(), sizeof(int64_t) * p->L, hipMemcpyHostToDevice)) !=
                hipSuccess)
                return P3_ERR_DEVICE;
            p->release = p->next_release;
        }
        p->mode = p->next_mode;
        p->policy = p->next_policy;
        p->pending_mode = false;
    }
    if (p->pending_tuning) {
        if (p->next_wgs_per_cu) p->wgs_per_cu = p->next_wgs_per_cu;
        if (p->next_reserved_cus >= 0) p->reserved_cus = p->next_reserved_cus;
        if (p->next_lean >= 0 && p->next_lean != p->lean) {
            p->lean = p->next_lean;
            if (!p->tile_elems)
                if (int rc = alloc_queue(p)) return rc;      // the default tile differs between the builds
        }
        p->next_lean = -1;
        if (p->next_tile_elems && p->next_tile_elems != p->tile_elems) {
            const int32_t old = p->tile_elems;
            p->tile_elems = p->next_tile_elems;
            if (int rc = alloc_queue(p)) {
                p->tile_elems = old;
                (void)alloc_queue(p);
                p->pending_tuning = false;
                return rc;
            }
        }
        p->pending_tuning = false;
        if (int rc = size_grid(p)) return rc;
    }
    return P3_OK;
}

// ---------------------------------------------------------------- iteration ----
int p3_begin_iter(p3_plan_t* p) {
    if (!p) return P3_ERR_ARG;
    if (!p->bound) return P3_ERR_STATE;
    if (HIPC(hipSetDevice(p->device)) != hipSuccess) return P3_ERR_DEVICE;
    if (p->live_issued && p->in_flight) {
        if (HIPC(hipEventQuery(p->ev_iter[p->last_slot])) != hipSuccess) return P3_ERR_STATE;   // live drain still running
        p->in_flight = false;
    }
    if (int rc = apply_pending(p)) return rc;
    std::lock_guard<std::mutex> lk(p->mu_host);
    p->iter_seq += 1;
    // The mark ring holds kEventRing iterations: before reusing a quarter, the
    // drains that read it (two iterations back) must be over.
    const int slot = static_cast<int>(p->iter_seq % kEventRing);
    const int old = static_cast<int>((p->iter_seq + kEventRing - 2) % kEventRing);
    if (p->ev_iter_used[old]) {
        if (HIPC(hipEventSynchronize(p->ev_iter[old])) != hipSuccess) return P3_ERR_DEVICE;
        p->ev_iter_used[old] = false;
    }
    p->ev_iter_used[slot] = false;
    p->epoch_base = p->marks_total;
    p->drained_upto = p->marks_total;
    std::fill(p->marked.begin(), p->marked.end(), 0);
    std::fill(p->t_seen_done_ns.begin(), p->t_seen_done_ns.end(), 0);
    p->first_drain = true;
    p->stream_marks = false;
    p->live_issued = false;
    p->iter_open = true;
    reinterpret_cast<std::atomic<uint32_t>*>(&p->hs->abort_flag)->store(0u, std::memory_order_release);
    p->hs->worker_status = P3D_OK;
    return P3_OK;
}

// A layer of which a sharded plan owns no slice is done, as far as this plan goes, the moment it is
// marked; the device still gets the mark (it counts marks) and folds nothing for it.
static void finish_empty_layer(p3_plan_s* p, int32_t layer, int64_t t) {
    if (p->layers[layer].count != 0) return;
    p->t_seen[layer] = 0;
    p->t_done[layer] = 0;
    p->t_seen_done_ns[layer] = t;
    reinterpret_cast<std::atomic<uint32_t>*>(&p->done_flag[layer])->store(p->iter_seq, std::memory_order_release);
}

int p3_mark_ready(p3_plan_t* p, int32_t layer) {
    if (!p) return P3_ERR_ARG;
    const int64_t t = now_ns();
    std::lock_guard<std::mutex> lk(p->mu_host);
    if (!p->bound || !p->iter_open) return P3_ERR_STATE;
    if (layer < 0 || layer >= p->L) return P3_ERR_RANGE;
    if (p->marked[layer]) return P3_ERR_ALREADY;
    p->marked[layer] = 1;
    p->t_mark_ns[layer] = t;
    // one 64-bit store: the entry carries its own position, which is what makes it valid
    reinterpret_cast<std::atomic<unsigned long long>*>(&p->mark_log[p->marks_total % p->mark_cap])
        ->store(mark_entry(p->marks_total, layer), std::memory_order_release);
    p->marks_total += 1;
    reinterpret_cast<std::atomic<uint64_t>*>(&p->hs->n_marks)->store(p->marks_total, std::memory_order_release);
    finish_empty_layer(p, layer, t);
    return P3_OK;
}

int p3_mark_ready_many(p3_plan_t* p, const int32_t* layers, int32_t n) {
    if (!p || n < 0 || (n > 0 && !layers)) return P3_ERR_ARG;
    for (int32_t i = 0; i < n; ++i)
        if (int rc = p3_mark_ready(p, layers[i])) return rc;
    return P3_OK;
}

// The mark as the last operation of a stream: one lane stores the entry into the pinned log.
__global__ void p3_mark_kernel(unsigned long long* slot, unsigned long long entry) {
    __hip_atomic_store(slot, entry, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

int p3_mark_ready_on_stream(p3_plan_t* p, int32_t layer, void* producer_stream) {
    if (!p) return P3_ERR_ARG;
    const int64_t t = now_ns();
    std::lock_guard<std::mutex> lk(p->mu_host);
    if (!p->bound || !p->iter_open) return P3_ERR_STATE;
    if (layer < 0 || layer >= p->L) return P3_ERR_RANGE;
    if (p->marked[layer]) return P3_ERR_ALREADY;
    if (HIPC(hipSetDevice(p->device)) != hipSuccess) return P3_ERR_DEVICE;
    // the position in mark order is taken now; the entry appears when the stream gets there
    hipLaunchKernelGGL(p3_mark_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(producer_stream),
                       &p->mark_log[p->marks_total % p->mark_cap], mark_entry(p->marks_total, layer));
    if (HIPC(hipGetLastError()) != hipSuccess) return P3_ERR_DEVICE;
    p->marked[layer] = 1;
    p->t_mark_ns[layer] = t;
    p->stream_marks = true;
    p->stream_ops = true;
    p->marks_total += 1;
    reinterpret_cast<std::atomic<uint64_t>*>(&p->hs->n_marks)->store(p->marks_total, std::memory_order_release);
    finish_empty_layer(p, layer, t);
    return P3_OK;
}

// The consumer's side of the same idea: a stream waits, on the device, until the layer's done flag
// carries this iteration's number.  One lane polls the pinned flag; the wait is bounded.
// (The clock is read with volatile inline assembly: as an intrinsic the read has no operands and may be
// moved out of the loop, which would make the time limit a constant.)
__device__ __forceinline__ unsigned long long wait_clock_now() {
    unsigned long long t;
    asm volatile("s_memrealtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(t) : : "memory");
    return t;
}

__global__ void p3_wait_kernel(const uint32_t* flag, uint32_t want, unsigned long long limit_ticks,
                               uint32_t* expired) {
    const unsigned long long t0 = wait_clock_now();
    while (__hip_atomic_load(flag, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_SYSTEM) != want) {
        if (wait_clock_now() - t0 > limit_ticks) {
            __hip_atomic_store(expired, want, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            break;
        }
        __builtin_amdgcn_s_sleep(64);
    }
}

int p3_wait_layer_on_stream(p3_plan_t* p, int32_t layer, void* consumer_stream, int32_t timeout_ms) {
    if (!p) return P3_ERR_ARG;
    if (!p->bound || !p->iter_open) return P3_ERR_STATE;
    if (layer < 0 || layer >= p->L) return P3_ERR_RANGE;
    if (HIPC(hipSetDevice(p->device)) != hipSuccess) return P3_ERR_DEVICE;
    const int32_t ms = timeout_ms >= 0 ? timeout_ms : p->watchdog_ms;
    hipLaunchKernelGGL(p3_wait_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(consumer_stream),
                       &p->done_flag[layer], p->iter_seq,
                       static_cast<unsigned long long>(ms) * static_cast<unsigned long long>(p->clock_khz),
                       p->wait_expired);
    if (HIPC(hipGetLastError()) != hipSuccess) return P3_ERR_DEVICE;
    p->stream_ops = true;
    return P3_OK;
}

int p3_stream_wait_expired(p3_plan_t* p) {
    if (!p) return P3_ERR_ARG;
    if (!p->bound) return P3_ERR_STATE;
    const uint32_t v = reinterpret_cast<std::atomic<uint32_t>*>(p->wait_expired)->load(std::memory_order_acquire);
    return (v != 0u && v == p->iter_seq) ? 1 : 0;
}

int p3_drain(p3_plan_t* p, void* hip_stream) {
    if (!p) return P3_ERR_ARG;
    if (!p->bound || !p->iter_open) return P3_ERR_STATE;
    if (HIPC(hipSetDevice(p->device)) != hipSuccess) return P3_ERR_DEVICE;
    uint64_t limit;
    {
        std::lock_guard<std::mutex> lk(p->mu_host);
        limit = p->marks_total;
    }
    if (p->mode == P3_MODE_LIVE) {
        if (p->live_issued) return P3_ERR_STATE;
    } else if (limit == p->drained_upto) {
        return P3_OK;             // nothing newly marked: nothing to claim
    }

    P3DrainArgs a;
    std::memset(&a, 0, sizeof a);
    a.slices = p->d_slices;
    a.layers = p->d_layers;
    a.release = p->d_release;
    a.bitmap = p->d_bitmap;
    a.layer_state = p->d_layer_state;
    a.runq = p->d_runq;
    a.order = p->d_order;
    a.epoch = p->d_epoch;
    // the iteration's first drain moves on to the set of counts that the iteration before it cleared
    const int32_t count_set = p->first_drain ? (p->count_set ^ 1) : p->count_set;
    a.layer_done = p->d_layer_done + static_cast<size_t>(count_set) * static_cast<size_t>(p->L);
    a.layer_req = p->d_layer_req + static_cast<size_t>(count_set) * static_cast<size_t>(p->L);
    a.layer_done_next = p->d_layer_done + static_cast<size_t>(count_set ^ 1) * static_cast<size_t>(p->L);
    a.layer_req_next = p->d_layer_req + static_cast<size_t>(count_set ^ 1) * static_cast<size_t>(p->L);
    a.fifo = p->d_fifo;
    a.t_seen_dev = p->d_t_seen;
    a.ctl = p->d_ctl;
    a.hs = p->hs;
    a.mark_log = p->mark_log;
    a.done_flag = p->done_flag;
    a.t_seen = p->t_seen;
    a.t_done = p->t_done;
    a.w = p->w;
    a.m = p->m;
    a.arena_elems = p->arena;
    a.K = p->K;
    a.L = p->L;
    a.n_words = (p->K + 63) / 64;
    a.mark_cap = p->mark_cap;
    a.run_cap = p->run_cap;
    a.tile_elems = tile_of_plan(p);
    a.tiles_per_full_slice = tiles_of(p->S < INT32_MAX ? p->S : INT32_MAX, a.tile_elems);
    a.epoch_base = p->epoch_base;
    a.epoch_limit = limit;
    a.watchdog_ticks = static_cast<uint64_t>(p->watchdog_ms) * static_cast<uint64_t>(p->clock_khz);
    a.lookahead = p->lookahead > 0 ? static_cast<uint32_t>(p->lookahead) : 2u * p->grid;
    a.iter_seq = p->iter_seq;
    a.mode = p->mode;
    a.policy = p->policy;
    a.iter_begin = p->first_drain ? 1 : 0;
    a.n_blocks = p->grid;
    a.W = p->W;
    a.lr = p->lr;
    a.mu = p->mu;
    a.rescale = p->rescale;
    a.wd = p->wd;
    a.n_inline = 0;
    if (p->mode != P3_MODE_LIVE && !p->stream_marks && limit - p->drained_upto <= P3_INLINE_MARKS) {
        std::lock_guard<std::mutex> lk(p->mu_host);
        a.n_inline = static_cast<int32_t>(limit - p->drained_upto);
        for (int32_t i = 0; i < a.n_inline; ++i)
            a.inline_marks[i] = static_cast<int32_t>(
                p->mark_log[(p->drained_upto + static_cast<uint64_t>(i)) % p->mark_cap] & 0xffffffffull);
    }
    // What the selector's first step will claim follows from these marks alone when the rule is the paper's:
    // every earlier drain of the iteration has claimed all that was ready to it (a SNAPSHOT drain ends when
    // nothing ready is left), so the lowest-numbered slices of the newly marked layers come next.  Their leading
    // runs go along with the launch, so that no workgroup waits for the first publication.  (Not after an abort:
    // the drain it stopped may have left ready slices behind.  One cut short by its watchdog would be noticed by
    // the selector's comparison and reported as an error.)
    a.n_first = 0;
    const bool aborted = reinterpret_cast<std::atomic<uint32_t>*>(&p->hs->abort_flag)->load(std::memory_order_acquire) != 0u;
    if (a.n_inline > 0 && !aborted && p->mode == P3_MODE_SNAPSHOT && p->policy == P3_POLICY_PRIORITY && p->persistent)
        a.n_first = p3_first_step_runs(*p, a.inline_marks, a.n_inline, p->lean ? P3_BLOCK_LEAN : P3_BLOCK, a.first_runs,
                                       P3_INLINE_RUNS);

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    ProfPair* pp = nullptr;
    if (p->prof_on) {
        if (p->prof_used == p->prof_pool.size()) {
            ProfPair n;
            if (HIPC(hipEventCreate(&n.start)) != hipSuccess || HIPC(hipEventCreate(&n.stop)) != hipSuccess) return P3_ERR_DEVICE;
            p->prof_pool.push_back(n);
        }
        pp = &p->prof_pool[p->prof_used];
        if (HIPC(hipEventRecord(pp->start, st)) != hipSuccess) return P3_ERR_DEVICE;
    }
    const auto launch = p->lean ? p3_launch_drain_lean : p3_launch_drain;
    if (HIPC(static_cast<hipError_t>(launch(&a, &p->grads, p->dtype, (p->mode == P3_MODE_LIVE || p->persistent) ? 1 : 0, p->grid, st))) != hipSuccess)
        return P3_ERR_DEVICE;
    if (pp) {
        if (HIPC(hipEventRecord(pp->stop, st)) != hipSuccess) return P3_ERR_DEVICE;
        p->prof_used += 1;
    }
    const int slot = static_cast<int>(p->iter_seq % kEventRing);
    if (HIPC(hipEventRecord(p->ev_iter[slot], st)) != hipSuccess) return P3_ERR_DEVICE;
    p->ev_iter_used[slot] = true;
    p->last_slot = slot;
    p->in_flight = true;
    p->first_drain = false;
    p->count_set = count_set;
    p->drained_upto = limit;
    if (p->mode == P3_MODE_LIVE) p->live_issued = true;
    return P3_OK;
}

int p3_abort(p3_plan_t* p) {
    if (!p) return P3_ERR_ARG;
    if (!p->bound) return P3_ERR_STATE;
    reinterpret_cast<std::atomic<uint32_t>*>(&p->hs->abort_flag)->store(1u, std::memory_order_release);
    return P3_OK;
}

int p3_sync(p3_plan_t* p, int32_t timeout_ms) {
    if (!p) return P3_ERR_ARG;
    if (!p->bound) return P3_ERR_STATE;
    if (HIPC(hipSetDevice(p->device)) != hipSuccess) return P3_ERR_DEVICE;
    bool timed_out = false;
    if (int rc = wait_idle(p, timeout_ms, &timed_out)) return rc;
    // note layers whose completion the host now sees
    const int64_t t = now_ns();
    for (int32_t l = 0; l < p->L; ++l)
        if (p->t_seen_done_ns[l] == 0 &&
            reinterpret_cast<std::atomic<uint32_t>*>(&p->done_flag[l])->load(std::memory_order_acquire) == p->iter_seq)
            p->t_seen_done_ns[l] = t;
    if (timed_out) return P3_ERR_TIMEOUT;
    // an inconsistency the kernel found in its own bookkeeping (selector) or in a queue record (worker)
    if (p->hs->last_iter == p->iter_seq && (p->hs->last_status == P3D_OVERFLOW || p->hs->worker_status == P3D_OVERFLOW))
        return P3_ERR_DEVICE;
    if (p->live_issued && p->hs->last_iter == p->iter_seq &&
        (p->hs->last_status != P3D_OK || p->hs->last_claimed != static_cast<uint32_t>(p->K)))
        return P3_ERR_INCOMPLETE;
    if (p->hs->last_iter == p->iter_seq && (p->hs->last_status != P3D_OK || p->hs->worker_status != P3D_OK))
        return P3_ERR_INCOMPLETE;     // a snapshot/ticked drain was stopped by abort or its watchdog
    return P3_OK;
}

int p3_poll(p3_plan_t* p) {
    if (!p) return P3_ERR_ARG;
    if (!p->bound) return P3_ERR_STATE;
    if (!p->in_flight) return P3_OK;
    const hipError_t e = hipEventQuery(p->ev_iter[p->last_slot]);
    if (e == hipErrorNotReady) return P3_ERR_TIMEOUT;
    if (HIPC(e) != hipSuccess) return P3_ERR_DEVICE;
    p->in_flight = false;
    return P3_OK;
}

int p3_wait_layer(p3_plan_t* p, int32_t layer, int32_t timeout_ms) {
    if (!p) return P3_ERR_ARG;
    if (!p->bound || !p->iter_open) return P3_ERR_STATE;
    if (layer < 0 || layer >= p->L) return P3_ERR_RANGE;
    const uint32_t want = p->iter_seq;
    std::atomic<uint32_t>* flag = reinterpret_cast<std::atomic<uint32_t>*>(&p->done_flag[layer]);
    const int64_t t0 = now_ns();
    for (;;) {
        if (flag->load(std::memory_order_acquire) == want) {
            if (p->t_seen_done_ns[layer] == 0) p->t_seen_done_ns[layer] = now_ns();
            return P3_OK;
        }
        const int64_t waited = now_ns() - t0;
        if (timeout_ms >= 0 && waited > static_cast<int64_t>(timeout_ms) * 1000000) return P3_ERR_TIMEOUT;
        // the first 200 us are polled flat out (this is the latency the caller is after); a longer
        // wait gives the core to others between looks
        if (waited > 200000) std::this_thread::yield();
    }
}

static int32_t copy_log(p3_plan_t* p, const int32_t* d_src, int32_t* out, int32_t cap) {
    if (!p || !out || cap < 0) return P3_ERR_ARG;
    if (!p->bound) return P3_ERR_STATE;
    if (HIPC(hipSetDevice(p->device)) != hipSuccess) return P3_ERR_DEVICE;
    if (int rc = wait_idle(p, p->live_issued ? p->watchdog_ms + 1000 : -1, nullptr)) return rc;
    if (p->first_drain) return 0;                       // nothing drained in this iteration
    if (p->hs->last_iter != p->iter_seq) return P3_ERR_DEVICE;
    int32_t n = static_cast<int32_t>(p->hs->last_claimed);
    if (n > p->K) return P3_ERR_DEVICE;
    if (n > cap) return P3_ERR_RANGE;
    if (n > 0 && HIPC(hipMemcpy(out, d_src, sizeof(int32_t) * n, hipMemcpyDeviceToHost)) != hipSuccess)
        return P3_ERR_DEVICE;
    return n;
}

int32_t p3_query_order(p3_plan_t* p, int32_t* out, int32_t cap) {
    const int32_t n = copy_log(p, p ? p->d_order : nullptr, out, cap);
    if (n > 0 && p->n_shards > 1)                      // the device logs the plan's own numbering
        for (int32_t i = 0; i < n; ++i) {
            if (out[i] < 0 || out[i] >= p->K) return P3_ERR_DEVICE;
            out[i] = p->global_id[static_cast<size_t>(out[i])];
        }
    return n;
}

int32_t p3_query_trace(p3_plan_t* p, int32_t* epoch_seen, int32_t cap) {
    return copy_log(p, p ? p->d_epoch : nullptr, epoch_seen, cap);
}

int p3_layer_latency_ns(p3_plan_t* p, int32_t layer, int64_t* host_ns, int64_t* dev_ns) {
    if (!p) return P3_ERR_ARG;
    if (!p->bound) return P3_ERR_STATE;
    if (layer < 0 || layer >= p->L) return P3_ERR_RANGE;
    if (reinterpret_cast<std::atomic<uint32_t>*>(&p->done_flag[layer])->load(std::memory_order_acquire) != p->iter_seq)
        return P3_ERR_STATE;
    if (host_ns) {
        if (p->t_seen_done_ns[layer] == 0) return P3_ERR_STATE;
        *host_ns = p->t_seen_done_ns[layer] - p->t_mark_ns[layer];
    }
    if (dev_ns) {
        const uint64_t ticks = p->t_done[layer] - p->t_seen[layer];
        *dev_ns = static_cast<int64_t>(ticks * 1000000ull / static_cast<uint64_t>(p->clock_khz));
    }
    return P3_OK;
}

int p3_layer_timeline_ns(p3_plan_t* p, int32_t layer, int64_t* seen_ns, int64_t* done_ns) {
    if (!p) return P3_ERR_ARG;
    if (!p->bound) return P3_ERR_STATE;
    if (layer < 0 || layer >= p->L) return P3_ERR_RANGE;
    if (int rc = wait_idle(p, p->live_issued ? p->watchdog_ms + 1000 : -1, nullptr)) return rc;
    if (reinterpret_cast<std::atomic<uint32_t>*>(&p->done_flag[layer])->load(std::memory_order_acquire) != p->iter_seq)
        return P3_ERR_STATE;
    const uint64_t t0 = p->hs->t_sel_enter;
    auto ns = [&](uint64_t t) {
        const int64_t ticks = static_cast<int64_t>(t - t0);          // two's complement: earlier stamps come out negative
        return ticks * 1000000ll / static_cast<int64_t>(p->clock_khz);
    };
    if (seen_ns) *seen_ns = ns(p->t_seen[layer]);
    if (done_ns) *done_ns = ns(p->t_done[layer]);
    return P3_OK;
}

int p3_drain_status(p3_plan_t* p, int32_t* selector_status, int32_t* worker_status, int32_t* phase,
                    int32_t* claimed) {
    if (!p) return P3_ERR_ARG;
    if (!p->bound) return P3_ERR_STATE;
    if (selector_status) *selector_status = static_cast<int32_t>(p->hs->last_status);
    if (worker_status) *worker_status = static_cast<int32_t>(p->hs->worker_status);
    if (phase) *phase = static_cast<int32_t>(p->hs->phase);
    if (claimed) *claimed = static_cast<int32_t>(p->hs->last_claimed);
    return P3_OK;
}

int p3_selector_timeline_ns(p3_plan_t* p, int64_t* first_publish_ns, int64_t* finished_ns) {
    if (!p) return P3_ERR_ARG;
    if (!p->bound) return P3_ERR_STATE;
    if (int rc = wait_idle(p, p->live_issued ? p->watchdog_ms + 1000 : -1, nullptr)) return rc;
    const uint64_t t0 = p->hs->t_sel_enter;
    auto ns = [&](uint64_t t) {
        return t >= t0 ? static_cast<int64_t>((t - t0) * 1000000ull / static_cast<uint64_t>(p->clock_khz)) : -1;
    };
    if (first_publish_ns) *first_publish_ns = p->hs->t_sel_first_pub ? ns(p->hs->t_sel_first_pub) : -1;
    if (finished_ns) *finished_ns = ns(p->hs->t_sel_final);
    return P3_OK;
}

int p3_profile_enable(p3_plan_t* p, int32_t on) {
    if (!p) return P3_ERR_ARG;
    if (!p->bound) return P3_ERR_STATE;
    if (int rc = wait_idle(p, p->live_issued ? p->watchdog_ms + 1000 : -1, nullptr)) return rc;
    try {
        collect_profile(p);
    } catch (const std::bad_alloc&) {
        return P3_ERR_NOMEM;
    }
    if (on) {
        p->prof_ms = 0.0;
        p->prof_launches = 0;
        p->prof_each.clear();
    }
    p->prof_on = on != 0;
    return P3_OK;
}

int p3_profile_read(p3_plan_t* p, double* total_ms, int32_t* launches, float* each_ms, int32_t cap) {
    if (!p || cap < 0 || (cap > 0 && !each_ms)) return P3_ERR_ARG;
    if (!p->bound) return P3_ERR_STATE;
    if (int rc = wait_idle(p, p->live_issued ? p->watchdog_ms + 1000 : -1, nullptr)) return rc;
    try {
        collect_profile(p);
    } catch (const std::bad_alloc&) {
        return P3_ERR_NOMEM;
    }
    if (total_ms) *total_ms = p->prof_ms;
    if (launches) *launches = p->prof_launches;
    const size_t n = p->prof_each.size() < static_cast<size_t>(cap) ? p->prof_each.size() : static_cast<size_t>(cap);
    for (size_t i = 0; i < n; ++i) each_ms[i] = p->prof_each[i];
    return P3_OK;
}

}  // extern "C"

// ------------------------------------------------- a drain that allocates nothing ----
// For callers that cannot allocate (code under HIP graph capture, tight serving loops,
// harnesses that forbid hipMalloc): one iteration -- marks, then a SNAPSHOT drain -- whose
// control data (slice and layer tables, ready bitmap, work queue, counters, flags, the
// kernel's mailbox) lives in one file-scope device array instead of buffers p3_bind
// allocated.  Every call on a GPU shares that GPU's array.

#define P3_STATIC_TABLE_CHUNK 128     // layers described per launch of the table kernel

namespace {

struct StaticScratch {
    // ---- cleared at the start of every call (everything up to `layers`) ----
    P3Ctl ctl;
    P3HostShared hs;                                  // the kernel's mailbox; device memory here
    unsigned long long bitmap[P3_STATIC_MAX_SLICES / 64];
    unsigned long long mark_log[64];                  // never read: the marks travel with the launch
    unsigned long long layer_done[P3_STATIC_MAX_LAYERS];
    uint64_t t_seen_dev[P3_STATIC_MAX_LAYERS];
    uint64_t t_seen[P3_STATIC_MAX_LAYERS];
    uint64_t t_done[P3_STATIC_MAX_LAYERS];
    int64_t release[P3_STATIC_MAX_LAYERS];
    uint32_t layer_req[P3_STATIC_MAX_LAYERS];
    uint32_t done_flag[P3_STATIC_MAX_LAYERS];
    int32_t fifo[P3_STATIC_MAX_LAYERS];
    uint8_t layer_state[P3_STATIC_MAX_LAYERS];
    // ---- rewritten by the table kernel / the selector before they are read ----
    alignas(128) P3LayerDev layers[P3_STATIC_MAX_LAYERS];
    int32_t epoch[P3_STATIC_MAX_SLICES];
    P3SliceDev slices[P3_STATIC_MAX_SLICES];
    P3Run runq[P3_STATIC_MAX_SLICES];
};

constexpr size_t kStaticBytes = (sizeof(StaticScratch) + 255) / 256 * 256;      // about 310 KB
static_assert(P3_STATIC_MAX_LAYERS <= P3_INLINE_MARKS, "the marks of a call travel with the launch arguments");
static_assert(P3_STATIC_MAX_SLICES <= P3_LDS_BM_WORDS * 64 && P3_STATIC_MAX_LAYERS <= P3_LDS_LAYERS,
              "the selector keeps bitmap and layer states in LDS");

}  // namespace

// In host code this name is a stand-in, not a device address: host code uses the pointer that
// hipGetSymbolAddress returns for the current device (static_state below), never the name.
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

namespace {

struct StaticDevice {
    StaticScratch* ptr = nullptr;      // this device's copy of `scratch`
    int num_cu = 0;
    int clock_khz = 100000;
    bool ready = false;
};
constexpr int kMaxDevices = 64;
StaticDevice g_static[kMaxDevices];
std::mutex g_static_mu;

// Set-up, once per device, with that device current.
int static_state(StaticDevice** out) {
    int dev = 0;
    if (HIPC(hipGetDevice(&dev)) != hipSuccess) return P3_ERR_DEVICE;
    if (dev < 0 || dev >= kMaxDevices) return P3_ERR_RANGE;
    std::lock_guard<std::mutex> lk(g_static_mu);
    StaticDevice& d = g_static[dev];
    if (!d.ready) {
        void* ptr = nullptr;
        if (HIPC(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))) != hipSuccess || !ptr) return P3_ERR_DEVICE;
        int cus = 0, khz = 0;
        if (HIPC(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess || cus < 1)
            return P3_ERR_DEVICE;
        if (HIPC(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev)) == hipSuccess && khz > 0)
            d.clock_khz = khz;
        d.ptr = static_cast<StaticScratch*>(ptr);
        d.num_cu = cus;
        d.ready = true;
    }
    *out = &d;
    return P3_OK;
}

// What must start at zero does: a fill kernel, not hipMemsetAsync, so that the call may be captured.
__global__ void p3_static_clear_kernel(StaticScratch* s, uint32_t n_words_bitmap) {
    uint32_t* w = reinterpret_cast<uint32_t*>(s);
    const uint32_t n = static_cast<uint32_t>(offsetof(StaticScratch, layers) / 4);
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) w[i] = 0u;
    __syncthreads();
    if (blockIdx.x == 0 && threadIdx.x == 0) {      // block 0 covers the control block's words itself (grid of 1 below)
        s->ctl.final_runs = P3_NONE;
        s->ctl.lo_word = n_words_bitmap;
    }
}

struct StaticTableArgs {
    int64_t elems[P3_STATIC_TABLE_CHUNK];
    int64_t offset[P3_STATIC_TABLE_CHUNK];
    int32_t first[P3_STATIC_TABLE_CHUNK];
    int32_t count[P3_STATIC_TABLE_CHUNK];
    int64_t S;
    int32_t base;         // index of the chunk's first layer
    int32_t n;            // layers in this chunk
};

// The slice table (Sec. 4.2) written on the device: workgroup b describes layer base + b.
__global__ void p3_static_table_kernel(StaticScratch* s, const StaticTableArgs a) {
    const int b = blockIdx.x;
    if (b >= a.n) return;
    const int layer = a.base + b;
    if (threadIdx.x == 0) {
        P3LayerDev ld;
        ld.first = a.first[b];
        ld.count = a.count[b];
        ld.elems = a.elems[b];
        s->layers[layer] = ld;
    }
    for (int i = threadIdx.x; i < a.count[b]; i += blockDim.x) {
        P3SliceDev sl;
        sl.start = a.offset[b] + static_cast<int64_t>(i) * a.S;
        const int64_t left = a.elems[b] - static_cast<int64_t>(i) * a.S;
        sl.len = static_cast<int32_t>(left < a.S ? left : a.S);
        sl.layer = layer;
        sl.layer_slices = a.count[b];
        sl.index_in_layer = i;
        sl.layer_elems = a.elems[b];
        s->slices[a.first[b] + i] = sl;
    }
}

// What the caller gets back: slices claimed, how selector and workers ended, layers published.
__global__ void p3_static_result_kernel(const StaticScratch* s, int32_t L, uint32_t iter_seq, int32_t* result) {
    __shared__ int n_done;
    if (threadIdx.x == 0) n_done = 0;
    __syncthreads();
    int mine = 0;
    for (int l = threadIdx.x; l < L; l += blockDim.x)
        if (__hip_atomic_load(&s->done_flag[l], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) == iter_seq) mine += 1;
    atomicAdd(&n_done, mine);
    __syncthreads();
    if (threadIdx.x == 0) {
        result[0] = static_cast<int32_t>(s->hs.last_claimed);
        result[1] = static_cast<int32_t>(s->hs.last_status);
        result[2] = static_cast<int32_t>(s->hs.worker_status);
        result[3] = n_done;
    }
}

}  // namespace

extern "C" int p3_drain_static(const p3_plan_t* p, int32_t W, const void* const* grads, int32_t grad_dtype,
                               float* weights, float* momentum, float lr, float mu, float rescale, float wd,
                               const int32_t* ready_layers, int32_t n_ready, int32_t* order_out,
                               int32_t* result_out, void* hip_stream) {
    if (!p || !grads || !weights || !momentum || !order_out || !result_out) return P3_ERR_ARG;
    if (n_ready < 0 || (n_ready > 0 && !ready_layers)) return P3_ERR_ARG;
    if (grad_dtype != P3_GRAD_FP32 && grad_dtype != P3_GRAD_BF16) return P3_ERR_ARG;
    if (W < 1 || W > P3_MAX_WORKERS) return P3_ERR_RANGE;
    if (p->n_shards != 1) return P3_ERR_ARG;
    if (p->L > P3_STATIC_MAX_LAYERS || p->K > P3_STATIC_MAX_SLICES) return P3_ERR_RANGE;   // beyond the static array
    auto misaligned = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) != 0; };
    if (misaligned(weights) || misaligned(momentum)) return P3_ERR_ARG;
    for (int32_t k = 0; k < W; ++k)
        if (!grads[k] || misaligned(grads[k])) return P3_ERR_ARG;
    uint8_t seen[P3_STATIC_MAX_LAYERS] = {0};
    for (int32_t i = 0; i < n_ready; ++i) {
        const int32_t l = ready_layers[i];
        if (l < 0 || l >= p->L) return P3_ERR_RANGE;
        if (seen[l]) return P3_ERR_ALREADY;
        seen[l] = 1;
    }
    const int32_t tile = P3_BLOCK * 4;
    const int64_t tiles = total_tiles(p, tile);
    if (tiles > INT32_MAX - 65536) return P3_ERR_RANGE;

    StaticDevice* d = nullptr;
    if (int rc = static_state(&d)) return rc;
    StaticScratch* s = d->ptr;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int32_t n_words = (p->K + 63) / 64;

    hipLaunchKernelGGL(p3_static_clear_kernel, dim3(1), dim3(1024), 0, st, s, static_cast<uint32_t>(n_words));
    if (HIPC(hipGetLastError()) != hipSuccess) return P3_ERR_DEVICE;
    for (int32_t base = 0; base < p->L; base += P3_STATIC_TABLE_CHUNK) {
        StaticTableArgs t;
        std::memset(&t, 0, sizeof t);
        t.S = p->S;
        t.base = base;
        t.n = p->L - base < P3_STATIC_TABLE_CHUNK ? p->L - base : P3_STATIC_TABLE_CHUNK;
        for (int32_t i = 0; i < t.n; ++i) {
            t.elems[i] = p->layers[base + i].elems;
            t.offset[i] = p->offset[base + i];
            t.first[i] = p->layers[base + i].first;
            t.count[i] = p->layers[base + i].count;
        }
        hipLaunchKernelGGL(p3_static_table_kernel, dim3(static_cast<unsigned>(t.n)), dim3(256), 0, st, s, t);
        if (HIPC(hipGetLastError()) != hipSuccess) return P3_ERR_DEVICE;
    }
    if (n_ready > 0) {
        P3DrainArgs a;
        std::memset(&a, 0, sizeof a);
        a.slices = s->slices;
        a.layers = s->layers;
        a.release = s->release;
        a.bitmap = s->bitmap;
        a.layer_state = s->layer_state;
        a.runq = s->runq;
        a.order = order_out;
        a.epoch = s->epoch;
        a.layer_done = s->layer_done;
        a.layer_req = s->layer_req;
        a.fifo = s->fifo;
        a.t_seen_dev = s->t_seen_dev;
        a.ctl = &s->ctl;
        a.hs = &s->hs;
        a.mark_log = s->mark_log;
        a.done_flag = s->done_flag;
        a.t_seen = s->t_seen;
        a.t_done = s->t_done;
        a.w = weights;
        a.m = momentum;
        a.arena_elems = p->arena;
        a.K = p->K;
        a.L = p->L;
        a.n_words = n_words;
        a.mark_cap = 64;
        a.run_cap = P3_STATIC_MAX_SLICES;
        a.tile_elems = tile;
        a.tiles_per_full_slice = tiles_of(p->S < INT32_MAX ? p->S : INT32_MAX, tile);
        a.epoch_base = 0;
        a.epoch_limit = static_cast<uint64_t>(n_ready);
        a.watchdog_ticks = 10000ull * static_cast<uint64_t>(d->clock_khz);
        unsigned grid = static_cast<unsigned>(d->num_cu);
        if (tiles < static_cast<int64_t>(grid)) grid = tiles < 2 ? 2u : static_cast<unsigned>(tiles);
        a.lookahead = 2u * grid;
        a.iter_seq = 1u;
        a.mode = P3_MODE_SNAPSHOT;
        a.policy = P3_POLICY_PRIORITY;
        a.iter_begin = 1;
        a.n_blocks = grid;
        a.W = W;
        a.lr = lr;
        a.mu = mu;
        a.rescale = rescale;
        a.wd = wd;
        a.n_inline = n_ready;
        for (int32_t i = 0; i < n_ready; ++i) a.inline_marks[i] = ready_layers[i];
        a.n_first = p3_first_step_runs(*p, a.inline_marks, a.n_inline, P3_BLOCK, a.first_runs, P3_INLINE_RUNS);
        P3GradPtrs gp;
        std::memset(&gp, 0, sizeof gp);
        for (int32_t k = 0; k < W; ++k) gp.p[k] = grads[k];
        if (HIPC(static_cast<hipError_t>(p3_launch_drain(&a, &gp, grad_dtype, 1, grid, st))) != hipSuccess)
            return P3_ERR_DEVICE;
    }
    hipLaunchKernelGGL(p3_static_result_kernel, dim3(1), dim3(256), 0, st, s, p->L, 1u, result_out);
    if (HIPC(hipGetLastError()) != hipSuccess) return P3_ERR_DEVICE;
    return P3_OK;
}
