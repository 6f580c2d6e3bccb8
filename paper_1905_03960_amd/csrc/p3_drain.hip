// Persistent drain kernel for gfx950 (MI355X): the P3 server's consumer loop
// (paper Sec. 4.2) as one launch.
//
//   workgroup 0  = the selector.  It folds newly marked layers into a ready
//                  bitmap (one bit per slice, bit index = global slice id =
//                  urgency rank), repeatedly takes the lowest set bits with
//                  popcount / prefix-sum / find-first-set across a wavefront,
//                  logs them as the claim order, groups the claimed slices into
//                  runs (slices of one layer that follow each other in memory)
//                  and appends the runs to a queue in global memory.
//   every workgroup (the selector too, once it is done) = a worker.  It draws
//                  the next tile number, finds the tile's run in its LDS copy of
//                  the queue, streams the W gradient copies plus weights and
//                  momentum of the tile (one quad of parameters per lane), sums
//                  the copies in fixed worker order in registers, applies the
//                  momentum and weight update, stores, and counts the tile
//                  against its layer; a layer whose count is complete gets its
//                  done flag after the L2 caches have been written back.
//
// The stream is HBM-bound (W*b + 16 bytes and W+3 flops per parameter): no
// matrix cores, LDS only for the queue copy and the selector's staging.
//
// Arithmetic per element, one binary32 rounding per operation, never fused:
//   s = ((g0 + g1) + ...) + g_{W-1};  s = rescale*s; [s = s + wd*w];
//   m' = mu*m - lr*s;  w' = w + m'
// This file must be compiled with -ffp-contract=off; the pragma below repeats it.

#include <hip/hip_runtime.h>

#include "p3_internal.h"

#pragma clang fp contract(off)

// Build parameters (p3_drain_lean.hip sets them and includes this file): a namespace for everything below, so
// that two builds can live in one library; the names of the two entry points; attributes of the kernels; how
// many loads a lane issues ahead of the one it is folding in.
#ifdef P3_NS
#define P3_NS_BEGIN namespace P3_NS {
#define P3_NS_END }
#define P3_NS_Q P3_NS::
#else
#define P3_NS_BEGIN
#define P3_NS_END
#define P3_NS_Q
#endif
#ifndef P3_LAUNCH_SYM
#define P3_LAUNCH_SYM p3_launch_drain
#define P3_OCCUPANCY_SYM p3_drain_occupancy
#endif
#ifndef P3_KERNEL_ATTR
#define P3_KERNEL_ATTR
#endif
#ifndef P3_LOADS_AHEAD
#define P3_LOADS_AHEAD 1
#endif

static_assert(P3_INLINE_RUNS <= P3_RUN_CACHE, "the runs handed over with the launch go into the ring");
static_assert(sizeof(P3DrainArgs) + sizeof(P3GradPtrs) <= 4096, "the launch arguments of a kernel are limited to 4 KB");

P3_NS_BEGIN

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define P3_AGENT __HIP_MEMORY_SCOPE_AGENT
#define P3_SYSTEM __HIP_MEMORY_SCOPE_SYSTEM

// "Is this lane number n?" through an opaque copy of the lane id, so that the
// compiler sees every single-lane section as guarded by a condition of its own.
// When two sections share one condition it may merge their control flow across
// a loop's back edge and give the remaining lanes a private loop around the
// workgroup barriers -- on a SIMT machine without independent lane progress
// those lanes then spin while the leader lane never runs again.
__device__ __forceinline__ bool lane_is(int id, int n) {
    asm volatile("" : "+v"(id));
    return id == n;
}

// Values every lane of a wavefront holds alike, moved to scalar registers: the
// compiler then knows they are uniform (scalar branches, scalar address bases).
__device__ __forceinline__ uint32_t uni(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int32_t uni(int32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ unsigned long long uni(unsigned long long v) {
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v >> 32));
    return (static_cast<unsigned long long>(hi) << 32) | lo;
}

__device__ __forceinline__ unsigned long long read_lane64(unsigned long long v, int l) {
    const uint32_t lo = __builtin_amdgcn_readlane(static_cast<uint32_t>(v), l);
    const uint32_t hi = __builtin_amdgcn_readlane(static_cast<uint32_t>(v >> 32), l);
    return (static_cast<unsigned long long>(hi) << 32) | lo;
}

// "Do not look at this value before this point": the result of a memory
// operation issued earlier is given a new name here, so that the moves to scalar
// registers that consume it (and the wait they imply) cannot be scheduled back
// to where the operation was issued.
__device__ __forceinline__ void pin_here(uint32_t& v) { asm volatile("" : "+v"(v) : : "memory"); }
__device__ __forceinline__ void pin_here(unsigned long long& v) { asm volatile("" : "+v"(v) : : "memory"); }

// Wait until every vector-memory operation this wavefront has issued is complete: loads have
// returned, stores and atomics have been acknowledged by the L2 of this XCD.  A workgroup-scope
// fence does NOT do this on gfx950 (all wavefronts of a workgroup share one L2, so the compiler
// emits no wait for it, and none at a barrier either): wherever a barrier is followed by a count,
// a flag or a write-back that speaks for the stores of the whole workgroup, every wavefront runs
// this wait before the barrier.
__device__ __forceinline__ void wait_vm_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// The device's constant-rate clock (100 MHz), read where the program says and every time it says: as an
// intrinsic the read may be moved out of a loop by the compiler (it has no operands), which would turn
// every time limit in this file into a constant.  Costs about as much as a trip to memory.
__device__ __forceinline__ uint64_t clock_now() {
    uint64_t t;
    asm volatile("s_memrealtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(t) : : "memory");
    return t;
}

// Wait for this wavefront's LDS (and scalar-memory) operations only.
__device__ __forceinline__ void wait_lds_done() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// Hyper-parameters as the kernel sees them.  Whether weight decay takes part is
// a compile-time property of the kernel: a run-time test between the loads and
// the arithmetic of every vector was measured to cost 12 % of the stream's
// bandwidth (it splits the block the scheduler pipelines over).  `rescale` needs
// no test at all: multiplying by 1.0f returns its operand bit for bit.
template <bool WD>
struct HyperT {
    static constexpr bool has_wd = WD;
    float lr, mu, rescale, wd;
};

// ------------------------------------------------------------- arithmetic ----
template <class H>
__device__ __forceinline__ void sgd_step(f32x4 s, f32x4& w, f32x4& m, const H& h) {
    s = h.rescale * s;
    if constexpr (H::has_wd) {
        f32x4 d = h.wd * w;
        s = s + d;
    }
    f32x4 a = h.mu * m;
    f32x4 b = h.lr * s;
    m = a - b;
    w = w + m;
}

template <class H>
__device__ __forceinline__ void sgd_step1(float s, float& w, float& m, const H& h) {
    s = h.rescale * s;
    if constexpr (H::has_wd) {
        float d = h.wd * w;
        s = s + d;
    }
    float a = h.mu * m;
    float b = h.lr * s;
    m = a - b;
    w = w + m;
}

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// Stores of updated weights and momentum are written THROUGH the L2 of the
// writing XCD (sc1) with a streaming hint (nt): each of the 8 XCDs has its own
// L2, and a parameter is only "published" (Sec. 4.2) once it has left it.
// Writing through costs nothing here -- every byte goes to HBM once anyway --
// whereas writing back on demand (an agent-scope release fence per tile) walks
// the whole L2 each time and was measured at 7x the kernel time.
// 128-bit stores go through a raw buffer descriptor over the tile, the form
// that lets the cache policy be stated; out-of-range offsets would be dropped.
#define P3_BUF_FLAGS 0x00020000      // gfx9 raw buffer, 32-bit data format
#define P3_AUX_SC1_NT (16 | 2)       // sc1 | nt

__device__ __forceinline__ void store_out(__amdgpu_buffer_rsrc_t r, int byte_off, f32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, byte_off, 0, P3_AUX_SC1_NT);
}

__device__ __forceinline__ void store_out1(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, P3_AGENT);     // 32-bit store with sc1
}

// One element through the scalar path (unaligned heads and tails of a tile).
template <bool BF16, class H>
__device__ __forceinline__ void update_one(const P3GradPtrs& gp, int W, float* __restrict__ w,
                                           float* __restrict__ m, int64_t e, const H& h) {
    float s;
    if (BF16) {
        s = bf16_bits_to_f32(static_cast<const uint16_t*>(gp.p[0])[e]);
        for (int k = 1; k < W; ++k) s = s + bf16_bits_to_f32(static_cast<const uint16_t*>(gp.p[k])[e]);
    } else {
        s = static_cast<const float*>(gp.p[0])[e];
        for (int k = 1; k < W; ++k) s = s + static_cast<const float*>(gp.p[k])[e];
    }
    float wv = w[e], mv = m[e];
    sgd_step1(s, wv, mv, h);
    store_out1(m + e, mv);
    store_out1(w + e, wv);
}

// How a lane streams.  The loads of a step (W gradient vectors plus weights and
// momentum, for NV vectors) form one sequence, and the lane keeps exactly two of
// them in flight: it issues load i+1, then waits for load i and folds it in.
// More loads in flight do not buy bandwidth here -- 256 workgroups x 832 lanes x
// 2 x 16 bytes already cover the memory's bandwidth-delay product -- they only
// lengthen the queues in front of the HBM channels, and the measured rate falls
// from 6.65 TB/s (two in flight) to 6.1 TB/s (all twenty in flight).  Left to
// itself the compiler picks either schedule depending on the code around the
// loop, so the consumption points are pinned: an empty asm statement that
// "modifies" the value just loaded keeps its use, and with it the wait, in place;
// its memory clobber and the scheduling barrier keep the load issued just before
// it in front of that wait (otherwise the next load may sink below the wait and
// the arithmetic, and the lane has a single load in flight for a while: -2 %).
__device__ __forceinline__ void pin(f32x4& v) {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" : "+v"(v) : : "memory");
}
__device__ __forceinline__ void pin(u32x4& v) {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" : "+v"(v) : : "memory");
}

// Four bf16 values in two 32-bit words: in each word the low half is the even
// element.  Widening to binary32 is exact (the bits move up by 16).
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void pin(u32x2& v) {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" : "+v"(v) : : "memory");
}
__device__ __forceinline__ f32x4 widen_quad(u32x2 raw) {
    f32x4 v = {__uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xffff0000u), __uint_as_float(raw.y << 16),
               __uint_as_float(raw.y & 0xffff0000u)};
    return v;
}

// NV quads (4 consecutive fp32 elements each, P3_BLOCK quads apart) per lane.
// Sum of the W copies: left fold in worker order.
template <int WT, int NV, class H>
__device__ __forceinline__ void do_quads_f32(const P3GradPtrs& gp, int W, const f32x4* __restrict__ w4,
                                             const f32x4* __restrict__ m4, int64_t q, int local,
                                             __amdgpu_buffer_rsrc_t rw, __amdgpu_buffer_rsrc_t rm,
                                             const H& h) {
    f32x4 s[NV], wv[NV], mv[NV];
    if constexpr (WT > 0 && P3_LOADS_AHEAD > 1) {
        // the same sequence with P3_LOADS_AHEAD loads issued ahead of the one being folded in: a workgroup of
        // few lanes needs that many in flight to fill what its compute unit can keep outstanding
        constexpr int NL = (WT + 2) * NV;
        constexpr int D = P3_LOADS_AHEAD < NL ? P3_LOADS_AHEAD : NL - 1;
        f32x4 r[NL];
#pragma unroll
        for (int i = 0; i < NL; ++i) {
#pragma unroll
            for (int k = (i == 0 ? 0 : i + D); k <= i + D && k < NL; ++k) {
                const int st = k / NV;
                const int64_t at = q + (k % NV) * P3_BLOCK;
                r[k] = st < WT    ? __builtin_nontemporal_load(static_cast<const f32x4*>(gp.p[st]) + at)
                       : st == WT ? __builtin_nontemporal_load(w4 + at)
                                  : __builtin_nontemporal_load(m4 + at);
            }
            f32x4 cur = r[i];
            pin(cur);
            const int st = i / NV, u = i % NV;
            if (st == 0) s[u] = cur;
            else if (st < WT) s[u] = s[u] + cur;
            else if (st == WT) wv[u] = cur;
            else mv[u] = cur;
        }
    } else if constexpr (WT > 0) {
        // sequence position i: stream i / NV (gradient copies, then weights, then momentum), vector i % NV
        constexpr int NL = (WT + 2) * NV;
        f32x4 nxt = __builtin_nontemporal_load(static_cast<const f32x4*>(gp.p[0]) + q);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            f32x4 cur = nxt;
            if (i + 1 < NL) {
                const int st = (i + 1) / NV;
                const int64_t at = q + ((i + 1) % NV) * P3_BLOCK;
                nxt = st < WT    ? __builtin_nontemporal_load(static_cast<const f32x4*>(gp.p[st]) + at)
                      : st == WT ? __builtin_nontemporal_load(w4 + at)
                                 : __builtin_nontemporal_load(m4 + at);
            }
            pin(cur);
            const int st = i / NV, u = i % NV;
            if (st == 0) s[u] = cur;
            else if (st < WT) s[u] = s[u] + cur;
            else if (st == WT) wv[u] = cur;
            else mv[u] = cur;
        }
    } else {
        f32x4 nxt = __builtin_nontemporal_load(static_cast<const f32x4*>(gp.p[0]) + q);
        for (int k = 0; k < W; ++k) {
#pragma unroll
            for (int u = 0; u < NV; ++u) {
                f32x4 cur = nxt;
                const bool more = (u + 1 < NV) || (k + 1 < W);
                const int kn = (u + 1 < NV || k + 1 >= W) ? k : k + 1;     // never indexes past the W-th pointer
                const int64_t at = q + ((u + 1) % NV) * P3_BLOCK;
                nxt = more ? __builtin_nontemporal_load(static_cast<const f32x4*>(gp.p[kn]) + at)
                           : __builtin_nontemporal_load(w4 + q);
                pin(cur);
                s[u] = (k == 0) ? cur : s[u] + cur;
            }
        }
#pragma unroll
        for (int i = 0; i < 2 * NV; ++i) {          // weights, then momentum
            f32x4 cur = nxt;
            if (i + 1 < 2 * NV) {
                const int64_t at = q + ((i + 1) % NV) * P3_BLOCK;
                nxt = (i + 1) < NV ? __builtin_nontemporal_load(w4 + at) : __builtin_nontemporal_load(m4 + at);
            }
            pin(cur);
            if (i < NV) wv[i] = cur;
            else mv[i - NV] = cur;
        }
    }
#pragma unroll
    for (int u = 0; u < NV; ++u) sgd_step(s[u], wv[u], mv[u], h);
    // Every load of the step has returned (the arithmetic needed them all), and with them -- the counter
    // is one for loads and stores -- every store this wavefront issued for earlier tiles has been
    // acknowledged.  The worker loop relies on that; the wait is stated here so that it does not depend on
    // how the compiler places its own.
    wait_vm_done();
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        store_out(rm, (local + u * P3_BLOCK) * 16, mv[u]);
        store_out(rw, (local + u * P3_BLOCK) * 16, wv[u]);
    }
}

// One quad per lane with bf16 gradients: 8 bytes per copy, 16 bytes each of weights
// and momentum, so that every instruction of a wavefront reads or writes one
// contiguous stretch (with one 128-bit gradient word per lane a lane owns 32
// contiguous bytes of weights, two half-used cache lines per instruction: measured
// at 4.0 instead of 6.7 TB/s).  The gradient loads are half as big as with fp32
// copies, so four instead of two are kept in flight: the same 32 bytes per lane.
template <int WT, class H>
__device__ __forceinline__ void do_quad_bf16(const P3GradPtrs& gp, int W, const f32x4* __restrict__ w4,
                                             const f32x4* __restrict__ m4, int64_t q, int local,
                                             __amdgpu_buffer_rsrc_t rw, __amdgpu_buffer_rsrc_t rm,
                                             const H& h) {
    constexpr int D = 3;                 // loads issued ahead of the one being folded in
    f32x4 s, wv, mv;
    if constexpr (WT > 0) {
        u32x2 r[WT];
#pragma unroll
        for (int i = 0; i < D && i < WT; ++i) r[i] = __builtin_nontemporal_load(static_cast<const u32x2*>(gp.p[i]) + q);
        if constexpr (WT < D) wv = __builtin_nontemporal_load(w4 + q);
        if constexpr (WT + 1 < D) mv = __builtin_nontemporal_load(m4 + q);
#pragma unroll
        for (int i = 0; i < WT; ++i) {
            if (i + D < WT) r[i + D] = __builtin_nontemporal_load(static_cast<const u32x2*>(gp.p[i + D]) + q);
            else if (i + D == WT) wv = __builtin_nontemporal_load(w4 + q);
            else if (i + D == WT + 1) mv = __builtin_nontemporal_load(m4 + q);
            u32x2 cur = r[i];
            pin(cur);
            if (i == 0) s = widen_quad(cur);
            else s = s + widen_quad(cur);
        }
    } else {
        // run-time worker count: a rotating window of three loads ahead
        u32x2 zero = {0u, 0u};
        u32x2 r0 = __builtin_nontemporal_load(static_cast<const u32x2*>(gp.p[0]) + q);
        u32x2 r1 = W > 1 ? __builtin_nontemporal_load(static_cast<const u32x2*>(gp.p[1]) + q) : zero;
        u32x2 r2 = W > 2 ? __builtin_nontemporal_load(static_cast<const u32x2*>(gp.p[2]) + q) : zero;
        for (int k = 0; k < W; ++k) {
            u32x2 r3 = k + 3 < W ? __builtin_nontemporal_load(static_cast<const u32x2*>(gp.p[k + 3]) + q) : zero;
            u32x2 cur = r0;
            pin(cur);
            s = (k == 0) ? widen_quad(cur) : s + widen_quad(cur);
            r0 = r1;
            r1 = r2;
            r2 = r3;
        }
        wv = __builtin_nontemporal_load(w4 + q);
        mv = __builtin_nontemporal_load(m4 + q);
    }
    pin(wv);
    pin(mv);
    sgd_step(s, wv, mv, h);
    wait_vm_done();                      // (as in do_quads_f32: earlier tiles' stores are acknowledged by now)
    store_out(rm, local * 16, mv);
    store_out(rw, local * 16, wv);
}

// Aggregate + update elements [start, start+n) of the arenas with one workgroup.
// 128-bit accesses on the aligned body, scalar accesses on the < VEC-element
// head and tail.  Lane i of the body touches vector i, i+256, ...: consecutive
// lanes read consecutive 16-byte words of each stream.
// Nothing but straight-line code may sit between the loads of a step and its
// arithmetic: a branch there (even a uniform one) was measured to cost 12 % of
// the stream's bandwidth.
template <int WT, bool BF16, class H>
__device__ __forceinline__ int32_t process_tile(const P3GradPtrs& gp, int W, float* __restrict__ w,
                                             float* __restrict__ m, int64_t start, int32_t n,
                                             const H& h) {
    constexpr int VEC = 4;                           // fp32 and bf16 gradients alike: one quad per lane
    const int tid = threadIdx.x;
    int32_t head = static_cast<int32_t>((VEC - (start & (VEC - 1))) & (VEC - 1));
    if (head > n) head = n;
    const int32_t nvec = (n - head) / VEC;
    const int32_t tail = n - head - nvec * VEC;
    const int64_t body = start + head;             // multiple of VEC
    const int64_t v0 = body / VEC;                 // first vector index
    const f32x4* __restrict__ w4 = reinterpret_cast<const f32x4*>(w);
    const f32x4* __restrict__ m4 = reinterpret_cast<const f32x4*>(m);
    // descriptors over exactly the aligned body of this tile (<= 4 MiB)
    const int body_bytes = nvec * VEC * 4;
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(w + body, 0, body_bytes, P3_BUF_FLAGS);
    const __amdgpu_buffer_rsrc_t rm = __builtin_amdgcn_make_buffer_rsrc(m + body, 0, body_bytes, P3_BUF_FLAGS);

    int32_t i = tid;
    if (!BF16) {
        // fp32: one quad per lane per step
        for (; i < nvec; i += P3_BLOCK) do_quads_f32<WT, 1>(gp, W, w4, m4, v0 + i, i, rw, rm, h);
    } else {
        // bf16: one quad per lane per step
        for (; i < nvec; i += P3_BLOCK) do_quad_bf16<WT>(gp, W, w4, m4, v0 + i, i, rw, rm, h);
    }
    // head on wavefront 0, tail on wavefront 1 (both < VEC elements)
    if (tid < head) update_one<BF16>(gp, W, w, m, start + tid, h);
    const int t2 = tid - 64;
    if (t2 >= 0 && t2 < tail) update_one<BF16>(gp, W, w, m, body + static_cast<int64_t>(nvec) * VEC + t2, h);
    return nvec;                                     // lanes below this number loaded and stored a quad
}

// --------------------------------------------------- completion of a layer ----
// Completion of a layer (Sec. 4.2: updated parameters go out as soon as they
// are written).  A tile's retire count is added once every store of the tile has
// been acknowledged, i.e. has reached the L2 of the XCD that ran the tile; the
// workgroup whose count completes a layer therefore knows that all the layer's
// data sits in (or beyond) the eight L2s, not yet that it is in memory.  Having
// every tile followed by an L2 write-back costs 70 % of the bandwidth (measured),
// so write-backs are made on demand, in rounds:
//   the completing workgroup opens round q = ++flush_req, notes q for the layer, and
//   raises `req` (and, for layer 0, `urgent`) on every XCD's own control line;
//   every leader reads its XCD's line once per tile, with the 128-bit load that
//   rides on the tile-number round trip, and while it waits for work;
//   the first leader of an XCD to see a round nobody has undertaken claims it (atomic
//   max on the line's `claim`), stamps the time, runs an agent-scope release fence --
//   the write-back of that XCD's L2 -- and then raises the line's `ack` to q; one
//   write-back costs the XCD 0.3 to 1.6 us of streaming (measured), so busy
//   workgroups leave P3_FLUSH_GAP_TICKS between two of them (a model with 161
//   layers would otherwise spend a fifth of its drain in them) and rounds that
//   open meanwhile are served together; a workgroup with nothing else to do
//   serves at once, and so does everybody for a round opened by layer 0, the
//   layer the next forward pass needs first;
//   whoever raised an ack (or left the loop) looks whether every XCD that has
//   workgroups in the loop has acknowledged q, and then writes the done flags
//   of all layers noted for rounds <= q (a compare-and-swap per layer picks the
//   one writer).
// Workgroups register with their XCD's line when the kernel starts; the last one to
// leave an XCD writes its L2 back and acknowledges all rounds to come.
// All words of this protocol are touched with atomic operations only.
struct FlushCtx {
    P3Ctl* ctl;
    uint32_t* layer_req;
    const uint64_t* t_seen_dev;
    uint64_t* t_seen;
    uint64_t* t_done;
    uint32_t* done_flag;
    uint32_t iter_seq;
    int32_t L;
};

__device__ __forceinline__ int xcd_of_this_wave() {
    // XCC_ID[3:0] of hardware register 20: the accelerator complex die (and with it the L2) this wavefront runs on
    return static_cast<int>(__builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 20)) & (P3_MAX_XCD - 1);
}

// Write the done flag of every layer whose round has been acknowledged by all XCDs in use.
__device__ __attribute__((noinline)) void publish_flushed(FlushCtx a, int lane) {
    uint32_t m = 0xffffffffu;
    if (lane < P3_MAX_XCD) {
        const uint32_t used = __hip_atomic_load(&a.ctl->xcd[lane].used, __ATOMIC_RELAXED, P3_AGENT);
        const uint32_t ack = __hip_atomic_load(&a.ctl->xcd[lane].ack, __ATOMIC_RELAXED, P3_AGENT);
        if (used != 0u) m = ack;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint32_t t = __shfl_xor(m, d, 64);
        m = t < m ? t : m;
    }
    for (int base = 0; base < a.L; base += 64) {
        const int l = base + lane;
        if (l < a.L) {
            uint32_t v = __hip_atomic_load(&a.layer_req[l], __ATOMIC_RELAXED, P3_AGENT);
            if (v != 0u && (v & P3_PUBLISHED) == 0u && v <= m) {
                if (__hip_atomic_compare_exchange_strong(&a.layer_req[l], &v, v | P3_PUBLISHED, __ATOMIC_RELAXED,
                                                         __ATOMIC_RELAXED, P3_AGENT)) {
                    a.t_seen[l] = __hip_atomic_load(&a.t_seen_dev[l], __ATOMIC_RELAXED, P3_AGENT);
                    a.t_done[l] = clock_now();
                    __hip_atomic_store(&a.done_flag[l], a.iter_seq, __ATOMIC_RELEASE, P3_SYSTEM);
                }
            }
        }
    }
}

// What a leader knows of the rounds from its XCD's line (one 128-bit load).
struct FlushView {
    uint32_t req, urgent, claim, time32;
};

__device__ __forceinline__ u32x4 load_flush_view(P3Ctl* ctl, int xcd) {
    // cache-bypassing (agent-scope) 128-bit load of the first four words of the XCD's line
    const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(&ctl->xcd[xcd], 0, 16, P3_BUF_FLAGS);
    return __builtin_amdgcn_raw_buffer_load_b128(r, 0, 0, 16 /* sc1 */);
}

__device__ __forceinline__ FlushView view_of(u32x4 v) {
    FlushView f;
    f.req = uni(v.x);
    f.urgent = uni(v.y);
    f.claim = uni(v.z);
    f.time32 = uni(v.w);
    return f;
}

// Is it this workgroup's turn to serve?  Busy workgroups hold back unless the last write-back of
// this L2 began long enough ago or a round of layer 0 is waiting.
__device__ __forceinline__ bool flush_due(const FlushView& f, bool idle) {
    if (f.req <= f.claim) return false;
    if (idle || f.urgent > f.claim) return true;
    return static_cast<uint32_t>(clock_now()) - f.time32 >= P3_FLUSH_GAP_TICKS;
}

// Round `want` is open: write this XCD's L2 back unless another of its workgroups has undertaken to.
__device__ __attribute__((noinline)) void serve_flush(FlushCtx a, uint32_t want, int xcd, int lane) {
    uint32_t c = 0u;
    if (lane_is(lane, 0)) c = __hip_atomic_fetch_max(&a.ctl->xcd[xcd].claim, want, __ATOMIC_RELAXED, P3_AGENT);
    if (uni(c) >= want) return;
    if (lane_is(lane, 0))
        __hip_atomic_store(&a.ctl->xcd[xcd].time32, static_cast<uint32_t>(clock_now()), __ATOMIC_RELAXED, P3_AGENT);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    uint32_t o = 0u;
    if (lane_is(lane, 0)) o = __hip_atomic_fetch_max(&a.ctl->xcd[xcd].ack, want, __ATOMIC_RELAXED, P3_AGENT);
    (void)uni(o);                                   // the acknowledgement has been performed
    publish_flushed(a, lane);
}

// This workgroup's retire count completed `layer`: open a write-back round for it.
__device__ __attribute__((noinline)) void complete_layer(FlushCtx a, int layer, int xcd, int lane) {
    uint32_t q = 0u, o = 0u;
    if (lane_is(lane, 0)) q = __hip_atomic_fetch_add(&a.ctl->flush_req, 1u, __ATOMIC_RELAXED, P3_AGENT);
    const uint32_t round = uni(q) + 1u;
    if (lane_is(lane, 0)) o = __hip_atomic_exchange(&a.layer_req[layer], round, __ATOMIC_RELAXED, P3_AGENT);
    (void)uni(o);                                   // the note has been performed before anyone can acknowledge for it
    // tell every XCD (lane x tells XCD x); the first layers are what the next forward pass needs first: their
    // rounds are served without the delay that busy workgroups otherwise leave between two write-backs
    uint32_t h = 0u;
    if (lane < P3_MAX_XCD) {
        h = __hip_atomic_fetch_max(&a.ctl->xcd[lane].req, round, __ATOMIC_RELAXED, P3_AGENT);
        if (layer < P3_URGENT_LAYERS)
            h += __hip_atomic_fetch_max(&a.ctl->xcd[lane].urgent, round, __ATOMIC_RELAXED, P3_AGENT);
    }
    (void)uni(h);
    const FlushView f = view_of(load_flush_view(a.ctl, xcd));
    if (flush_due(f, false)) serve_flush(a, f.req, xcd, lane);
    publish_flushed(a, lane);                       // in case every other XCD had acknowledged before the note was visible
}

// This workgroup's one retire count was the whole layer (the count stood at zero before it): every
// store of the layer came from this workgroup, so only this XCD's L2 can hold any of it -- it is
// written back here and the layer published at once, without a round among the XCDs.  Used for layer
// 0 only, the case of a first layer of a few thousand parameters, whose latency matters most: every
// write-back stalls its XCD for a microsecond or so, and a model with a hundred one-tile layers (the
// normalisation vectors of a ResNet) that wrote back for each of them lost 6 % of its drain to that;
// the other layers wait for a round like everybody else.
__device__ __attribute__((noinline)) void complete_alone(FlushCtx a, int layer, int lane) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    if (lane_is(lane, 0)) {
        __hip_atomic_store(&a.layer_req[layer], P3_PUBLISHED, __ATOMIC_RELAXED, P3_AGENT);
        a.t_seen[layer] = __hip_atomic_load(&a.t_seen_dev[layer], __ATOMIC_RELAXED, P3_AGENT);
        a.t_done[layer] = clock_now();
        __hip_atomic_store(&a.done_flag[layer], a.iter_seq, __ATOMIC_RELEASE, P3_SYSTEM);
    }
}

// Every workgroup of a launch registers with its XCD before it does anything else
// (workgroup 0 of a fused launch before it starts selecting), so the set of XCDs a
// round has to hear from is fixed when the first store is made.
// (The selecting workgroup does not wait here: its first act that others can see is a publication
// of the queue, which sits behind an agent-scope release fence of this same wavefront, and that
// fence waits for these two operations as for every other one -- one round trip less in front of
// the first publication.)
__device__ __forceinline__ void enter_xcd(P3Ctl* ctl, int xcd, int lane, bool wait) {
    uint32_t u = 0u, v = 0u;
    if (lane_is(lane, 0)) {
        u = __hip_atomic_exchange(&ctl->xcd[xcd].used, 1u, __ATOMIC_RELAXED, P3_AGENT);
        v = __hip_atomic_fetch_add(&ctl->xcd[xcd].live, 1u, __ATOMIC_RELAXED, P3_AGENT);
    }
    if (wait) {
        (void)uni(u);
        (void)uni(v);                              // performed before this workgroup stores anything
    }
}

// Leaving the worker loop.  While other workgroups of the XCD stay, any write-back they make
// for a later round begins after this workgroup's last retire count and so covers its stores.
// The workgroup that empties the XCD writes the L2 back itself and then acknowledges every
// round there will ever be: nothing is left in that L2 that a round would have to wait for.
// (No workgroup leaves before the queue is final, so workgroup 0 of a fused launch is in the
// worker loop, or about to enter it, when the others of its XCD leave.)
__device__ __attribute__((noinline)) void leave_loop(FlushCtx a, int xcd, int lane) {
    uint32_t o = 0u;
    if (lane_is(lane, 0)) o = __hip_atomic_fetch_add(&a.ctl->xcd[xcd].live, 0xffffffffu, __ATOMIC_RELAXED, P3_AGENT);
    if (uni(o) != 1u) return;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    uint32_t k = 0u;
    if (lane_is(lane, 0)) k = __hip_atomic_fetch_max(&a.ctl->xcd[xcd].ack, 0xffffffffu, __ATOMIC_RELAXED, P3_AGENT);
    (void)uni(k);
    publish_flushed(a, lane);
}

// ---------------------------------------------------------------- selector ----
struct SelectorLds {
    int32_t batch[P3_BATCH_MAX];           // claimed slice ids of this step, ascending
    // runs of this step (a run = claimed slices of one layer that follow each other in memory)
    int64_t run_elem0[P3_BATCH_MAX + 1];   // elements of the step before the run (exclusive prefix)
    int64_t run_start[P3_BATCH_MAX];       // arena offset of the run's first element
    int32_t run_layer[P3_BATCH_MAX];
    int64_t wave_elems[P3_WAVES];
    int32_t wave_cnt[P3_WAVES];
    // working copies of the ready bitmap and the layer states for the duration of a launch (when they fit):
    // folding marks and taking the lowest bits then cost LDS latencies instead of trips to memory
    unsigned long long bm[P3_LDS_BM_WORDS];
    uint8_t lstate[P3_LDS_LAYERS];
    P3LayerDev pre[P3_INLINE_MARKS];       // table entries of the layers whose marks came with the launch, in mark order
    int32_t nb;                            // slices in this step
    int32_t done;
    int32_t overflow;                      // set by a single-wavefront step that found the queue full
    uint32_t claimed;                      // order-log position of batch[0]
    uint32_t epoch;                        // marks observed when this step was selected
    uint32_t pub_runs;                     // queue position of this step's first run
    uint32_t pub_tiles;                    // number of this step's first tile
};

__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int t = __shfl_up(v, d, 64);
        if (lane >= d) v += t;
    }
    return v;
}

__device__ __forceinline__ long long wave_incl_scan_i64(long long v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        long long t = __shfl_up(v, d, 64);
        if (lane >= d) v += t;
    }
    return v;
}

__device__ __forceinline__ long long wave_min_i64(long long v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        long long t = __shfl_xor(v, d, 64);
        v = t < v ? t : v;
    }
    return v;
}

// Selector state kept in wavefront-uniform registers of wavefront 0.
struct SelState {
    uint32_t claimed, marks_applied, n_ready, lo_word, pending, pub_runs, pub_tiles, status;
    uint32_t fifo_head, fifo_tail, cur_next, cur_left;   // first-come-first-served policy
    long long clock;
};

__device__ __forceinline__ int wave_sum_i32(int v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint32_t t = __shfl_xor(v, d, 64);
        v = t < v ? t : v;
    }
    return v;
}

// All slices of a layer enter the ready set at once (Sec. 4.2).  Every active
// lane folds a layer of its own (the layers are distinct): it ORs the layer's
// bit range into the bitmap word by word.  The ORs are atomic because two small
// layers can share a word, and nobody waits for them individually: one wait
// after the call covers all of them, so folding 64 marks costs one trip to
// memory instead of 64.  The bitmap is only ever touched with atomic
// operations, so all accesses meet at the same level of the memory system.
// `pre`: the layer's table entry if it has been fetched already (else it is loaded here: a trip to memory).
// `now`: the device clock as read at the top of the selection round (reading it costs about as much as a
// trip to memory, so it is read once per round, not once per use).
__device__ __forceinline__ void fold_lanes(const P3DrainArgs& a, unsigned long long* bm, uint8_t* ls, bool active,
                                           int layer, SelState& st, const P3LayerDev* pre, uint64_t now) {
    int count = 0, first = 0, end = 0;
    uint32_t w0 = 0xffffffffu;
    if (active) {
        const P3LayerDev ld = pre ? *pre : a.layers[layer];
        first = ld.first;
        end = ld.first + ld.count;
        w0 = static_cast<uint32_t>(first >> 6);
        ls[layer] = P3L_RELEASED;
        // device memory (the selector never waits on the host link), written through for the worker that reads it
        __hip_atomic_store(&a.t_seen_dev[layer], now, __ATOMIC_RELAXED, P3_AGENT);
        count = ld.count;
    }
    // the words [from, to] of the range [first, end) that this lane ORs in, `step` apart
    auto or_words = [&](int first_, int end_, int from, int to, int step) {
        for (int wi = from; wi <= to; wi += step) {
            const int lo = (first_ > wi * 64 ? first_ : wi * 64) - wi * 64;
            const int hi = (end_ < wi * 64 + 64 ? end_ : wi * 64 + 64) - wi * 64;
            const unsigned long long ones = (hi - lo == 64) ? ~0ull : ((1ull << (hi - lo)) - 1ull);
            __hip_atomic_fetch_or(&bm[wi], ones << lo, __ATOMIC_RELAXED, P3_AGENT);
        }
    };
    // A layer of a few words is its lane's own business; a layer of many slices (small slices, or a
    // fully connected layer) would keep one lane busy for hundreds of dependent steps while 63 wait,
    // so the whole wavefront fills it, 64 words per step.
    const bool wide = active && ((end - 1) >> 6) - (first >> 6) >= 4;
    if (active && !wide) or_words(first, end, first >> 6, (end - 1) >> 6, 1);
    unsigned long long wides = __ballot(wide);
    const int lane = static_cast<int>(threadIdx.x) & 63;
    while (wides != 0ull) {
        const int src = __builtin_ctzll(wides);
        wides &= wides - 1ull;
        const int f = __shfl(first, src, 64), e = __shfl(end, src, 64);
        or_words(f, e, (f >> 6) + lane, (e - 1) >> 6, 64);
    }
    st.n_ready += static_cast<uint32_t>(wave_sum_i32(count));
    const uint32_t lo_new = wave_min_u32(w0);
    if (lo_new < st.lo_word) st.lo_word = lo_new;
}

// Take the `want` lowest set bits of the bitmap (ascending slice id = most
// urgent first), clear them, and write their indices to lds.batch[0..want).
// Requires want <= n_ready.  One wavefront; 64 bitmap words per step.
__device__ __forceinline__ int take_lowest(const P3DrainArgs& a, unsigned long long* bm, SelectorLds& lds, int want, int lane,
                                           SelState& st) {
    int nb = 0;
    uint32_t wi = st.lo_word;
    while (nb < want && wi < static_cast<uint32_t>(a.n_words)) {
        const uint32_t my = wi + lane;
        unsigned long long word = 0ull;
        if (my < static_cast<uint32_t>(a.n_words)) word = __hip_atomic_load(&bm[my], __ATOMIC_RELAXED, P3_AGENT);
        if (__ballot(word != 0ull) == 0ull) {      // nothing ready in these 4096 slices
            wi += 64;
            continue;
        }
        const int cnt = __popcll(word);
        const int incl = wave_incl_scan(cnt, lane);
        const int excl = incl - cnt;
        const int total = __shfl(incl, 63, 64);
        const int room = want - nb;
        int take = room - excl;
        take = take < 0 ? 0 : (take > cnt ? cnt : take);
        // Bit extraction, one word at a time with the wavefront's lanes on the word's 64 bits (a lane
        // walking its own word bit by bit made this the longest part of a selection step: 64 dependent
        // iterations).  Words that give nothing are skipped.
        unsigned long long rest = word;
        unsigned long long givers = __ballot(take > 0);
        while (givers != 0ull) {
            const int src = __builtin_ctzll(givers);
            givers &= givers - 1ull;
            const unsigned long long w_s = read_lane64(word, src);
            const int excl_s = __builtin_amdgcn_readlane(excl, src);
            const int take_s = __builtin_amdgcn_readlane(take, src);
            const bool set = ((w_s >> lane) & 1ull) != 0ull;
            const int rank = __popcll(w_s & ((1ull << lane) - 1ull));
            const bool mine = set && rank < take_s;
            if (mine) lds.batch[nb + excl_s + rank] = static_cast<int32_t>((wi + static_cast<uint32_t>(src)) * 64u + lane);
            const unsigned long long taken = __ballot(mine);
            if (lane == src) rest = word & ~taken;
        }
        if (take > 0) __hip_atomic_store(&bm[my], rest, __ATOMIC_RELAXED, P3_AGENT);
        if (total <= room) {                       // window emptied
            nb += total;
            wi += 64;
        } else {
            nb += room;
        }
    }
    st.lo_word = wi;
    st.n_ready -= static_cast<uint32_t>(nb);
    return nb;                                     // == want whenever n_ready matched the bitmap
}

// First-come-first-served policy (the baseline the paper argues against, Sec. 3: gradients are
// synchronised in the order backward produces them, layer by layer).  Layers are served whole
// in the order they became ready: in SNAPSHOT and LIVE mode the order of the marks (an arrival
// queue in memory), in TICKED mode ascending release tick, the later layer first among equal
// ticks (backward order).  Writes `want` (or fewer, if the ready layers run out) slice ids to
// lds.batch.  One wavefront.
__device__ __forceinline__ int take_fifo(const P3DrainArgs& a, uint8_t* ls, SelectorLds& lds, int want, int lane,
                                         SelState& st, uint64_t now) {
    int nb = 0;
    while (nb < want) {
        if (st.cur_left == 0u) {
            int nl = -1;
            if (a.mode == 2) {
                long long best = 0x7fffffffffffffffLL;
                int bl = -1;
                for (int base = 0; base < a.L; base += 64) {
                    const int l = base + lane;
                    if (l < a.L && ls[l] == P3L_PENDING) {
                        const long long r = a.release[l];
                        if (bl < 0 || r < best || (r == best && l > bl)) {
                            best = r;
                            bl = l;
                        }
                    }
                }
#pragma unroll
                for (int d = 32; d >= 1; d >>= 1) {
                    const long long ob = __shfl_xor(best, d, 64);
                    const int ol = __shfl_xor(bl, d, 64);
                    if (ol >= 0 && (bl < 0 || ob < best || (ob == best && ol > bl))) {
                        best = ob;
                        bl = ol;
                    }
                }
                nl = uni(bl);
                if (nl < 0) break;
                if (lane_is(lane, 0)) {
                    ls[nl] = P3L_RELEASED;
                    __hip_atomic_store(&a.t_seen_dev[nl], now, __ATOMIC_RELAXED, P3_AGENT);
                }
                st.pending -= 1u;
            } else {
                if (st.fifo_head == st.fifo_tail) break;
                nl = uni(__hip_atomic_load(&a.fifo[st.fifo_head], __ATOMIC_RELAXED, P3_AGENT));
                st.fifo_head += 1u;
            }
            st.cur_next = static_cast<uint32_t>(uni(a.layers[nl].first));
            st.cur_left = static_cast<uint32_t>(uni(a.layers[nl].count));
        }
        const int room = want - nb;
        const int take = static_cast<uint32_t>(room) < st.cur_left ? room : static_cast<int>(st.cur_left);
        for (int i = lane; i < take; i += 64) lds.batch[nb + i] = static_cast<int32_t>(st.cur_next) + i;
        nb += take;
        st.cur_next += static_cast<uint32_t>(take);
        st.cur_left -= static_cast<uint32_t>(take);
    }
    st.n_ready -= static_cast<uint32_t>(nb);
    return nb;
}

// Does run r of the first selection step (start rs, length rl, layer) differ from what the host handed the
// workers with the launch?  (Thread r asks; the step must have at least as many runs as were handed over.)
__device__ __forceinline__ bool first_run_differs(const P3DrainArgs& a, int r, int nruns, long long rs, long long rl,
                                                  int layer) {
    if (r >= a.n_first) return false;
    if (r >= nruns) return true;
    const P3FirstRun f = a.first_runs[r];
    return f.start != rs || static_cast<long long>(f.len) != rl || f.layer != layer;
}

__device__ void run_selector(const P3DrainArgs& a, SelectorLds& lds) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: whole wavefronts branch on it
    P3Ctl* ctl = a.ctl;

    const uint64_t t_entry = clock_now();
    // Memory ordering.  A store's acknowledgement (what `s_waitcnt vmcnt(0)` waits for; a
    // workgroup-scope fence waits for nothing here) only says that the store has reached the L2
    // of the issuing XCD; other XCDs see it once that L2 has written it back, and only an
    // agent-scope release fence waits for that (measured: a
    // flag stored after acknowledged write-through stores is seen by other workgroups before
    // the data).  So the selector raises `published` behind an agent-scope release fence -- one
    // L2 write-back per selection step.  The bitmap, the layer states and the selector's
    // counters are touched by this workgroup alone within a launch; launches are ordered by the
    // stream.  Counters shared with the workers are only ever touched with atomic operations,
    // which are performed at the memory side.
    const bool in_lds = a.n_words <= P3_LDS_BM_WORDS && a.L <= P3_LDS_LAYERS;
    unsigned long long* bm = in_lds ? lds.bm : a.bitmap;
    uint8_t* ls = in_lds ? lds.lstate : a.layer_state;
    if (in_lds && !a.iter_begin) {
        for (int i = tid; i < a.n_words; i += P3_BLOCK) bm[i] = a.bitmap[i];
        for (int i = tid; i < a.L; i += P3_BLOCK) ls[i] = a.layer_state[i];
    }
    if (a.iter_begin) {
        for (int i = tid; i < a.n_words; i += P3_BLOCK) bm[i] = 0ull;
        for (int i = tid; i < a.L; i += P3_BLOCK) {
            ls[i] = P3L_IDLE;
            // (the counts of THIS iteration were cleared by the first drain of the iteration before; what is
            // cleared here is the set the next iteration will count in)
            if (a.layer_done_next != nullptr) {
                __hip_atomic_store(&a.layer_done_next[i], 0ull, __ATOMIC_RELAXED, P3_AGENT);
                __hip_atomic_store(&a.layer_req_next[i], 0u, __ATOMIC_RELAXED, P3_AGENT);
            }
        }
        if (lane_is(tid, 0)) {
            ctl->claimed = 0u;
            ctl->marks_applied = 0u;
            ctl->n_ready = 0u;
            ctl->lo_word = static_cast<uint32_t>(a.n_words);
            ctl->pending = 0u;
            ctl->clock = 0;
            ctl->fifo_head = ctl->fifo_tail = 0u;
            ctl->cur_next = ctl->cur_left = 0u;
        }
    }
    // The table entries of the layers whose marks came with the launch are asked for now, all at once (one
    // thread per mark), so that the wait below covers them too: folding the marks then needs no trip to
    // memory (it used to take one per 64 marks, each behind the other).
    const bool pre_ok = a.n_inline > 0;
    P3LayerDev pre_mine;
    pre_mine.first = pre_mine.count = 0;
    pre_mine.elems = 0;
    if (pre_ok && tid < a.n_inline) {
        const int32_t l = a.inline_marks[tid];
        if (l >= 0 && l < a.L) pre_mine = a.layers[l];
    }
    wait_vm_done();                     // the table entries asked for above are here
    if (pre_ok && tid < a.n_inline) lds.pre[tid] = pre_mine;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();

    SelState st;
    if (a.iter_begin) {                 // what was just written above: no trip to memory for it
        st.claimed = st.marks_applied = st.n_ready = st.pending = 0u;
        st.lo_word = static_cast<uint32_t>(a.n_words);
        st.clock = 0;
        st.fifo_head = st.fifo_tail = st.cur_next = st.cur_left = 0u;
    } else {
        st.claimed = ctl->claimed;
        st.marks_applied = ctl->marks_applied;
        st.n_ready = ctl->n_ready;
        st.lo_word = ctl->lo_word;
        st.pending = ctl->pending;
        st.clock = ctl->clock;
        st.fifo_head = ctl->fifo_head;
        st.fifo_tail = ctl->fifo_tail;
        st.cur_next = ctl->cur_next;
        st.cur_left = ctl->cur_left;
    }
    st.pub_runs = 0u;
    st.pub_tiles = 0u;
    st.status = P3D_OK;
    const uint64_t t_start = t_entry;
    const uint32_t inline_first = st.marks_applied;   // first mark this drain folds
    const FlushCtx sel_fc = {a.ctl, a.layer_req, a.t_seen_dev, a.t_seen, a.t_done, a.done_flag, a.iter_seq, a.L};
    const int sel_xcd = xcd_of_this_wave();
    uint32_t rounds = 0u;
    // (Nothing is stored over the host link before the first publication: the release fence in front of a
    // publication waits for every store this wavefront has outstanding, and one to host memory takes longest.)
    if (lane_is(tid, 0)) lds.overflow = 0;

    for (;;) {
        if (wave == 0) {
            int budget = 0;
            bool done = false, gave_up = false, folded_now = false;
            // (1) fold newly visible marks, in mark order.  A mark is an entry of the pinned log that carries
            //     its own position; it may come from the host or from a stream, and it is taken when it and all
            //     marks before it are there.  SNAPSHOT/TICKED: the marks up to the drain call belong to this
            //     drain -- those the host made travel with the launch, one a stream still has to make is
            //     waited for (bounded by the watchdog).  LIVE: whatever has arrived.
            uint64_t lim = a.epoch_limit;
            if (a.mode == 1) lim = a.epoch_base + static_cast<uint64_t>(a.L);
            // the device clock, once per round (the first round makes do with the stamp taken at entry)
            const uint64_t t_round = rounds == 0u ? t_entry : clock_now();
            // LIVE: everything a round needs from outside the CU -- the next entries of the mark log and the
            // stop flag (both over the host link), this XCD's write-back line, the workers' tile counter -- is
            // asked for at once, one wait instead of four in a row (a selection step took 7.5 us, half of
            // it these round trips; the look-ahead the workers need grows with the length of a step).
            unsigned long long e_first = 0ull;
            uint32_t ab_first = 0u, tk_first = 0u;
            u32x4 fv_first = {0u, 0u, 0u, 0u};
            bool pre = a.mode == 1;
            if (pre) {
                const uint64_t base0 = a.epoch_base + st.marks_applied;
                if (base0 + static_cast<uint64_t>(lane) < lim)
                    e_first = __hip_atomic_load(&a.mark_log[(base0 + lane) % a.mark_cap], __ATOMIC_RELAXED, P3_SYSTEM);
                ab_first = __hip_atomic_load(&a.hs->abort_flag, __ATOMIC_RELAXED, P3_SYSTEM);
                fv_first = load_flush_view(ctl, sel_xcd);
                tk_first = __hip_atomic_load(&ctl->ticket, __ATOMIC_RELAXED, P3_AGENT);
            }
            // The mark log lives in host memory: fetch up to 64 entries per trip over the
            // host link (one per lane) instead of one trip per mark.
            while (a.epoch_base + st.marks_applied < lim) {
                const uint64_t base = a.epoch_base + st.marks_applied;
                int n_new = lim - base > 64 ? 64 : static_cast<int>(lim - base);
                int my_layer = -1;
                uint32_t pre_idx = 0u;
                if (a.n_inline > 0) {        // came with the launch: marks_applied counts from inline_marks[0]
                    if (lane < n_new) {
                        const uint32_t idx = st.marks_applied - inline_first + static_cast<uint32_t>(lane);
                        if (idx < static_cast<uint32_t>(a.n_inline)) {
                            my_layer = a.inline_marks[idx];
                            pre_idx = idx;
                        }
                    }
                } else {
                    bool there = false;
                    if (lane < n_new) {
                        const unsigned long long e =
                            pre ? e_first
                                : __hip_atomic_load(&a.mark_log[(base + lane) % a.mark_cap], __ATOMIC_RELAXED, P3_SYSTEM);
                        there = static_cast<uint32_t>(e >> 32) == static_cast<uint32_t>(base + lane + 1);
                        my_layer = static_cast<int32_t>(e & 0xffffffffull);
                    }
                    pre = false;                 // the entries asked for above were those at this position
                    // the leading entries that are there
                    const unsigned long long missing = ~__ballot(there);
                    const int lead = missing == 0ull ? 64 : __builtin_ctzll(missing);
                    n_new = lead < n_new ? lead : n_new;
                    if (lane >= n_new) my_layer = -1;
                    if (n_new == 0) {
                        if (a.mode == 1) break;                       // LIVE: nothing new now
                        // a mark that a stream has yet to make: wait for it, within the drain's time limit
                        if (clock_now() - t_start > a.watchdog_ticks ||
                            __hip_atomic_load(&a.hs->abort_flag, __ATOMIC_RELAXED, P3_SYSTEM) != 0u) {
                            gave_up = true;
                            break;
                        }
                        __builtin_amdgcn_s_sleep(32);
                        continue;
                    }
                }
                const bool ok = my_layer >= 0 && my_layer < a.L && ls[my_layer] == P3L_IDLE;
                if (a.policy == 1) {
                    // first come, first served: the layer joins the arrival queue (or, TICKED, the pending set)
                    const unsigned long long oks = __ballot(ok);
                    int cnt = 0;
                    if (ok) {
                        cnt = a.layers[my_layer].count;
                        if (a.mode == 2) {
                            ls[my_layer] = P3L_PENDING;
                        } else {
                            ls[my_layer] = P3L_RELEASED;
                            const uint32_t pos = st.fifo_tail + static_cast<uint32_t>(__popcll(oks & ((1ull << lane) - 1ull)));
                            __hip_atomic_store(&a.fifo[pos], my_layer, __ATOMIC_RELAXED, P3_AGENT);
                            __hip_atomic_store(&a.t_seen_dev[my_layer], t_round, __ATOMIC_RELAXED, P3_AGENT);
                        }
                    }
                    st.n_ready += static_cast<uint32_t>(wave_sum_i32(cnt));
                    if (a.mode == 2) st.pending += static_cast<uint32_t>(__popcll(oks));
                    else st.fifo_tail += static_cast<uint32_t>(__popcll(oks));
                } else if (a.mode == 2) {
                    if (ok) ls[my_layer] = P3L_PENDING;
                    st.pending += static_cast<uint32_t>(__popcll(__ballot(ok)));
                } else {
                    // (marks read over the host link: the stamp is taken now, the read of the clock hides behind
                    // the link's latency; marks that came with the launch carry the round's stamp)
                    fold_lanes(a, bm, ls, ok, my_layer, st, pre_ok ? &lds.pre[pre_idx] : nullptr,
                               a.n_inline > 0 ? t_round : clock_now());
                }
                st.marks_applied += static_cast<uint32_t>(n_new);
                folded_now = true;
                // the ORs have landed (a bitmap in LDS: nothing here waits for memory -- the stamps stored by
                // fold_lanes are covered by the release fence in front of the next publication)
                if (in_lds) wait_lds_done();
                else {
                    wait_vm_done();
                    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
                }
                // LIVE: look again only if this look came back full (then more marks may be waiting behind
                // it).  A host that marks layer after layer without a pause would otherwise keep this loop
                // going -- every look finds another mark or two -- and nothing would be claimed until the
                // last mark is in: what is ready is served while the rest arrives.
                if (a.mode == 1 && n_new < 64) break;
            }
            // a short first step gets the workers going; later steps amortise the publication
            // (as many slices as give every workgroup two tiles, at least what one wavefront groups on its own)
            // (a full step when the workers have been handed its leading runs with the launch: nobody waits for it)
            const int first_cap = a.n_first > 0 ? P3_BATCH_MAX : p3_first_step_slices(a.n_blocks, a.tiles_per_full_slice);
            const int batch_cap = st.pub_runs == 0u ? first_cap : P3_BATCH_MAX;
            // every mode: the host may ask the drain to stop, and no drain outlives its watchdog
            // (a read over the host link: every round in LIVE mode, where the drain waits on the
            // host anyway; every 8th round otherwise, and not before the first publication)
            uint32_t ab = ab_first;
            if (a.mode != 1 && ((rounds & 7u) == 7u || gave_up))
                ab = __hip_atomic_load(&a.hs->abort_flag, __ATOMIC_RELAXED, P3_SYSTEM);
            if (a.mode == 1) {
                // a LIVE selection lasts as long as the iteration: meanwhile this workgroup answers for
                // its XCD in the write-back rounds like any waiting workgroup (it may be the only one there)
                const FlushView fv = view_of(fv_first);
                if (flush_due(fv, true)) serve_flush(sel_fc, fv.req, sel_xcd, lane);
            }
            rounds += 1u;
            const bool expired = t_round - t_start > a.watchdog_ticks;
            // (2) decide how many slices may be claimed now
            if (ab != 0u || expired || gave_up) {
                done = true;
                st.status = ab != 0u ? P3D_ABORTED : P3D_WATCHDOG;
            } else if (a.mode == 2 && a.policy == 1) {
                // TICKED, first come first served: the order is that of the release ticks; no clock is needed
                budget = st.n_ready > static_cast<uint32_t>(batch_cap) ? batch_cap : static_cast<int>(st.n_ready);
                done = (st.n_ready == 0u);
            } else if (a.mode == 2) {
                // TICKED: release what the clock has reached; if nothing is ready jump to the next release
                long long next;
                for (;;) {
                    next = 0x7fffffffffffffffLL;
                    for (int base = 0; base < a.L; base += 64) {
                        const int l = base + lane;
                        bool rel = false;
                        if (l < a.L && ls[l] == P3L_PENDING) {
                            const long long r = a.release[l];
                            if (r <= st.clock) rel = true;
                            else if (r < next) next = r;
                        }
                        fold_lanes(a, bm, ls, rel, l, st, nullptr, t_round);
                        st.pending -= static_cast<uint32_t>(__popcll(__ballot(rel)));
                        if (in_lds) wait_lds_done();
                        else {
                            wait_vm_done();
                            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
                        }
                    }
                    next = wave_min_i64(next);
                    if (st.n_ready == 0u && st.pending > 0u) {
                        st.clock = next;
                        continue;
                    }
                    break;
                }
                long long b = st.n_ready;
                if (st.pending > 0u && next - st.clock < b) b = next - st.clock;
                budget = b > batch_cap ? batch_cap : static_cast<int>(b);
                done = (st.n_ready == 0u && st.pending == 0u);
            } else if (a.mode == 0) {
                budget = st.n_ready > static_cast<uint32_t>(batch_cap) ? batch_cap : static_cast<int>(st.n_ready);
                done = (st.n_ready == 0u);
            } else {
                // LIVE: stay at most `lookahead` tiles ahead of the workers
                if (st.claimed == static_cast<uint32_t>(a.K)) {
                    done = true;
                } else if (st.n_ready == 0u) {
                    __builtin_amdgcn_s_sleep(16);
                } else if (st.marks_applied == static_cast<uint32_t>(a.L)) {
                    // every layer has been marked: nothing more urgent can arrive any more, so there is no
                    // reason to hold claims back -- the rest of the iteration is claimed in full steps (the
                    // step that follows a mark stays short: what has just arrived is published sooner)
                    const int cap = folded_now ? 64 : batch_cap;
                    budget = st.n_ready > static_cast<uint32_t>(cap) ? cap : static_cast<int>(st.n_ready);
                } else {
                    const uint32_t tk = uni(tk_first);
                    const uint32_t ahead = st.pub_tiles > tk ? st.pub_tiles - tk : 0u;
                    if (ahead >= a.lookahead) {
                        __builtin_amdgcn_s_sleep(4);
                    } else {
                        uint32_t b = (a.lookahead - ahead) / static_cast<uint32_t>(a.tiles_per_full_slice);
                        if (b < 1u) b = 1u;
                        if (b > st.n_ready) b = st.n_ready;
                        budget = b > static_cast<uint32_t>(batch_cap) ? batch_cap : static_cast<int>(b);
                    }
                }
            }
            // (3) claim the `budget` most urgent ready slices
            if (budget > 0 && !done) {
                if (st.claimed + static_cast<uint32_t>(budget) > static_cast<uint32_t>(a.K)) {
                    done = true;                 // cannot happen with a consistent bitmap; never write past the log
                    st.status = P3D_OVERFLOW;
                    budget = 0;
                } else {
                    const int got = a.policy == 1 ? take_fifo(a, ls, lds, budget, lane, st, t_round)
                                                  : take_lowest(a, bm, lds, budget, lane, st);
                    if (got != budget) {         // bitmap and counter disagree: stop rather than spin
                        done = true;
                        st.status = P3D_OVERFLOW;
                    }
                    budget = got;
                    if (a.mode == 2 && a.policy == 0) st.clock += budget;
                }
            } else {
                budget = 0;
            }
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
            if (lane_is(lane, 0)) {
                lds.nb = budget;
                lds.done = done ? 1 : 0;
                lds.claimed = st.claimed;
                lds.epoch = st.marks_applied;
                lds.pub_runs = st.pub_runs;
                lds.pub_tiles = st.pub_tiles;
            }
        }
        __syncthreads();
        const int nb = lds.nb;
        if (nb == 0) {
            if (lds.done) break;
            __syncthreads();
            continue;
        }
        if (nb <= 64) {
            // (4') a step of at most one wavefront's worth of slices -- the usual size in LIVE mode, where the
            //      selector stays just ahead of the workers: wavefront 0 does what (4) below does, alone, with
            //      wavefront scans and no workgroup barrier (2.3 of a step's 7.5 us went into those)
            if (wave == 0) {
                int head = 0;
                long long len = 0;
                P3SliceDev sl;
                sl.start = 0;
                sl.layer = 0;
                if (lane < nb) {
                    const int g = lds.batch[lane];
                    sl = a.slices[g];
                    len = sl.len;
                    head = (lane > 0 && lds.batch[lane - 1] + 1 == g && sl.index_in_layer > 0) ? 0 : 1;
                    a.order[st.claimed + static_cast<uint32_t>(lane)] = g;
                    a.epoch[st.claimed + static_cast<uint32_t>(lane)] = static_cast<int32_t>(st.marks_applied);
                }
                const int h_incl = wave_incl_scan(head, lane);
                const long long e_incl = wave_incl_scan_i64(len, lane);
                const int nruns = __shfl(h_incl, 63, 64);
                const long long e_total = __shfl(e_incl, 63, 64);
                if (lane < nb && head) {
                    const int r = h_incl - 1;
                    lds.run_elem0[r] = e_incl - len;
                    lds.run_start[r] = sl.start;
                    lds.run_layer[r] = sl.layer;
                }
                if (lane_is(lane, 0)) lds.run_elem0[nruns] = e_total;
                __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");      // the lanes read each other's entries
                int c = 0, rlayer = 0;
                long long rs = 0, rl = 0;
                if (lane < nruns) {
                    rs = lds.run_start[lane];
                    rl = lds.run_elem0[lane + 1] - lds.run_elem0[lane];
                    rlayer = lds.run_layer[lane];
                    c = static_cast<int>((rs + rl - 1) / a.tile_elems - rs / a.tile_elems + 1);
                }
                const int c_incl = wave_incl_scan(c, lane);
                const int tb = __shfl(c_incl, 63, 64);
                bool fits = st.pub_runs + static_cast<uint32_t>(nruns) <= a.run_cap;
                if (st.pub_runs == 0u && a.n_first > 0 &&
                    __ballot(first_run_differs(a, lane, nruns, rs, rl, rlayer)) != 0ull)
                    fits = false;                      // the workers were handed something else: stop
                if (fits && lane < nruns) {
                    const uint32_t t0 = st.pub_tiles + static_cast<uint32_t>(c_incl - c);
                    unsigned long long* q =
                        reinterpret_cast<unsigned long long*>(&a.runq[st.pub_runs + static_cast<uint32_t>(lane)]);
                    __hip_atomic_store(q, static_cast<unsigned long long>(rs), __ATOMIC_RELAXED, P3_AGENT);
                    __hip_atomic_store(q + 1, static_cast<unsigned long long>(rl), __ATOMIC_RELAXED, P3_AGENT);
                    __hip_atomic_store(q + 2, (static_cast<unsigned long long>(static_cast<uint32_t>(rlayer)) << 32) |
                                                  static_cast<uint32_t>(rs % a.tile_elems), __ATOMIC_RELAXED, P3_AGENT);
                    __hip_atomic_store(q + 3, (static_cast<unsigned long long>(t0 + static_cast<uint32_t>(c)) << 32) | t0,
                                       __ATOMIC_RELAXED, P3_AGENT);
                }
                // the records are written back from this XCD's L2 before the queue grows
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
                st.claimed += static_cast<uint32_t>(nb);
                if (fits) {
                    const bool first = st.pub_runs == 0u;
                    st.pub_runs += static_cast<uint32_t>(nruns);
                    st.pub_tiles += static_cast<uint32_t>(tb);
                    if (lane_is(lane, 0)) {
                        __hip_atomic_store(&ctl->published, st.pub_runs, __ATOMIC_RELAXED, P3_AGENT);
                        if (first) {
                            a.hs->t_sel_enter = t_entry;
                            a.hs->t_sel_first_pub = clock_now();   // first growth
                            a.hs->phase = P3P_PUBLISHED;
                        }
                    }
                } else {
                    st.status = P3D_OVERFLOW;          // cannot happen: the queue has room for one run per slice
                    if (lane_is(lane, 0)) lds.overflow = 1;
                }
            }
            __syncthreads();                           // lds.nb has been read by everyone; the flag below is written
            if (uni(static_cast<uint32_t>(lds.overflow)) != 0u) break;
            continue;
        }
        // (4) log the claims, group the claimed slices into runs and append the runs to the queue
        //     (the whole workgroup; one claimed slice per thread)
        const uint32_t log_at = lds.claimed, epoch_now = lds.epoch, runs_at = lds.pub_runs, tiles_at = lds.pub_tiles;
        int head = 0;
        long long len = 0;
        P3SliceDev sl;
        sl.start = 0;
        sl.layer = 0;
        if (tid < nb) {
            const int g = lds.batch[tid];
            sl = a.slices[g];
            len = sl.len;
            // not a head: the slice claimed just before is this one's predecessor in the layer
            head = (tid > 0 && lds.batch[tid - 1] + 1 == g && sl.index_in_layer > 0) ? 0 : 1;
            a.order[log_at + tid] = g;
            a.epoch[log_at + tid] = static_cast<int32_t>(epoch_now);
        }
        const int h_incl = wave_incl_scan(head, lane);
        const long long e_incl = wave_incl_scan_i64(len, lane);
        if (lane_is(lane, 63)) {
            lds.wave_cnt[wave] = h_incl;
            lds.wave_elems[wave] = e_incl;
        }
        __syncthreads();
        int r_before = 0, nruns = 0;
        long long e_before = 0, e_total = 0;
#pragma unroll
        for (int v = 0; v < P3_WAVES; ++v) {
            const int wc = lds.wave_cnt[v];
            const long long we = lds.wave_elems[v];
            if (v < wave) {
                r_before += wc;
                e_before += we;
            }
            nruns += wc;
            e_total += we;
        }
        if (tid < nb && head) {
            const int r = r_before + h_incl - 1;
            lds.run_elem0[r] = e_before + e_incl - len;
            lds.run_start[r] = sl.start;
            lds.run_layer[r] = sl.layer;
        }
        if (lane_is(tid, 0)) lds.run_elem0[nruns] = e_total;
        __syncthreads();
        // thread r describes run r: its length, the grid cells (= tiles) it touches
        int c = 0;
        long long rs = 0, rl = 0;
        if (tid < nruns) {
            rs = lds.run_start[tid];
            rl = lds.run_elem0[tid + 1] - lds.run_elem0[tid];
            c = static_cast<int>((rs + rl - 1) / a.tile_elems - rs / a.tile_elems + 1);
        }
        const int c_incl = wave_incl_scan(c, lane);
        __syncthreads();                           // everyone has read the wave totals of the first scan
        if (lane_is(lane, 63)) lds.wave_cnt[wave] = c_incl;
        __syncthreads();
        int t_before = 0, tb = 0;
#pragma unroll
        for (int v = 0; v < P3_WAVES; ++v) {
            const int wc = lds.wave_cnt[v];
            if (v < wave) t_before += wc;
            tb += wc;
        }
        if (runs_at == 0u && a.n_first > 0 &&
            first_run_differs(a, tid, nruns, rs, rl, tid < nruns ? lds.run_layer[tid] : 0))
            lds.overflow = 1;                          // the workers were handed something else: stop
        __syncthreads();
        const bool fits = runs_at + static_cast<uint32_t>(nruns) <= a.run_cap && uni(static_cast<uint32_t>(lds.overflow)) == 0u;
        if (fits && tid < nruns) {
            const uint32_t t0 = tiles_at + static_cast<uint32_t>(t_before + c_incl - c);
            unsigned long long* q = reinterpret_cast<unsigned long long*>(&a.runq[runs_at + static_cast<uint32_t>(tid)]);
            __hip_atomic_store(q, static_cast<unsigned long long>(rs), __ATOMIC_RELAXED, P3_AGENT);
            __hip_atomic_store(q + 1, static_cast<unsigned long long>(rl), __ATOMIC_RELAXED, P3_AGENT);
            __hip_atomic_store(q + 2, (static_cast<unsigned long long>(static_cast<uint32_t>(lds.run_layer[tid])) << 32) |
                                          static_cast<uint32_t>(rs % a.tile_elems), __ATOMIC_RELAXED, P3_AGENT);
            __hip_atomic_store(q + 3, (static_cast<unsigned long long>(t0 + static_cast<uint32_t>(c)) << 32) | t0,
                               __ATOMIC_RELAXED, P3_AGENT);
        }
        // every wavefront's record stores have reached this XCD's L2 ...
        wait_vm_done();
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        if (wave == 0) {
            // ... and one wavefront has that L2 write them back before the queue grows
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            st.claimed += static_cast<uint32_t>(nb);
            if (fits) {
                const bool first = st.pub_runs == 0u;
                st.pub_runs += static_cast<uint32_t>(nruns);
                st.pub_tiles += static_cast<uint32_t>(tb);
                if (lane_is(lane, 0)) {
                    __hip_atomic_store(&ctl->published, st.pub_runs, __ATOMIC_RELAXED, P3_AGENT);
                    if (first) {                       // (stores over the host link once per launch, not per step)
                        a.hs->t_sel_enter = t_entry;
                        a.hs->t_sel_first_pub = clock_now();   // first growth
                        a.hs->phase = P3P_PUBLISHED;
                    }
                }
            } else {
                st.status = P3D_OVERFLOW;          // cannot happen: the queue has room for one run per slice
            }
        }
        if (!fits) break;
    }

    if (in_lds) {                       // the next drain of the iteration starts from these
        __syncthreads();
        for (int i = tid; i < a.n_words; i += P3_BLOCK) a.bitmap[i] = bm[i];
        for (int i = tid; i < a.L; i += P3_BLOCK) a.layer_state[i] = ls[i];
    }
    if (lane_is(tid, 0)) {
        ctl->claimed = st.claimed;
        ctl->marks_applied = st.marks_applied;
        ctl->n_ready = st.n_ready;
        ctl->lo_word = st.lo_word;
        ctl->pending = st.pending;
        ctl->clock = st.clock;
        ctl->fifo_head = st.fifo_head;
        ctl->fifo_tail = st.fifo_tail;
        ctl->cur_next = st.cur_next;
        ctl->cur_left = st.cur_left;
        a.hs->last_claimed = st.claimed;
        a.hs->last_status = st.status;
        a.hs->last_iter = a.iter_seq;
        __hip_atomic_store(&ctl->final_runs, st.pub_runs, __ATOMIC_RELAXED, P3_AGENT);
        if (st.pub_runs == 0u) {        // nothing was ever published: the stamps of a first publication were not written
            a.hs->t_sel_enter = t_entry;
            a.hs->t_sel_first_pub = 0;
        }
        a.hs->t_sel_final = clock_now();
        a.hs->phase = P3P_FINAL;
    }
    __syncthreads();
}

// ------------------------------------------------------------------ kernel ----
// Leader helpers of the worker loop -------------------------------------------
// Wavefront 0 is the leader.  All its lanes run the leader code with the same
// addresses, results are moved to scalar registers, and only read-modify-write
// operations and host stores are narrowed to lane 0.

// one lane takes the ticket; the value is left in a vector register (not waited for)
__device__ __forceinline__ uint32_t take_ticket(P3Ctl* ctl, int lane) {
    uint32_t k = 0u;
    if (lane_is(lane, 0)) k = __hip_atomic_fetch_add(&ctl->ticket, 1u, __ATOMIC_RELAXED, P3_AGENT);
    return k;
}

// (The out-of-line leader functions take what they need by value: handing them the
// kernel's argument block by reference would make every wavefront copy that block
// to its private stack when the kernel starts.)
struct QueueCtx {
    P3Ctl* ctl;
    const P3Run* runq;
    P3HostShared* hs;
    uint64_t watchdog_ticks;
    int64_t arena_elems;
    int32_t L;
    int32_t tile_elems;
};

struct Located {
    P3Run run;          // the run that holds the tile (found != 0)
    uint32_t r_next;    // runs below this index end at or before the tile
    uint32_t r_have;    // runs below this index have been copied to the LDS ring
    int32_t found;      // 0: the queue is complete (or the wait was given up) and has no such tile; 1: found;
                        // 2: the queue has not grown that far yet and the caller did not allow a wait
};

// Find the run that holds tile k.  Tile numbers only grow, so the search never
// goes back: runs [r_next, r_have) of the LDS ring are examined 64 at a time (one
// per lane), and when they are used up the ring is refilled from the queue in
// global memory -- waiting (bounded) for the queue to grow when the selector runs
// in the same launch (WAIT).  The queue entries are read with cache-bypassing
// loads: the selector wrote them through before raising `published`.
template <bool WAIT>
__device__ __attribute__((noinline)) Located locate_run(QueueCtx a, FlushCtx fc, int xcd, P3Run* ring, uint32_t k,
                                                        uint32_t r_next, uint32_t r_have, uint64_t t_enter, int lane,
                                                        bool may_wait) {
    Located out;
    out.run.start = 0;
    out.run.len = 0;
    out.run.grid_off = 0;
    out.run.layer = 0;
    out.run.tile0 = 0u;
    out.run.tile_end = 0u;
    out.found = 0;
    uint32_t looks = 0u;
    for (;;) {
        while (r_next < r_have) {
            const uint32_t r = r_next + static_cast<uint32_t>(lane);
            const bool in = r < r_have;
            uint32_t te = 0u;
            if (in) te = ring[r & (P3_RUN_CACHE - 1)].tile_end;
            const unsigned long long hit = __ballot(in && k < te);
            if (hit != 0ull) {
                const uint32_t rf = r_next + static_cast<uint32_t>(__builtin_ctzll(hit));
                const P3Run* e = &ring[rf & (P3_RUN_CACHE - 1)];
                out.run = *e;                                  // every lane reads the same entry
                out.r_next = rf + 1u;
                out.r_have = r_have;
                out.found = 1;
                return out;
            }
            r_next = r_have - r_next > 64u ? r_next + 64u : r_have;
        }
        // what a waiting workgroup needs from memory -- the queue's length, whether it is final, its XCD's
        // write-back line -- is asked for at once: one round trip per look, not three in a row
        uint32_t pub_v = __hip_atomic_load(&a.ctl->published, __ATOMIC_RELAXED, P3_AGENT);
        uint32_t fin_v = P3_NONE;
        u32x4 fv_v = {0u, 0u, 0u, 0u};
        if (WAIT) {
            fin_v = __hip_atomic_load(&a.ctl->final_runs, __ATOMIC_RELAXED, P3_AGENT);
            fv_v = load_flush_view(a.ctl, xcd);
        }
        const uint32_t pub = uni(pub_v);
        if (pub > r_have) {
            // r_next == r_have: everything in the ring is dead, the whole ring may be refilled
            const uint32_t upto = pub - r_have > P3_RUN_CACHE ? r_have + P3_RUN_CACHE : pub;
            for (uint32_t base = r_have; base < upto; base += 64u) {
                const uint32_t r = base + static_cast<uint32_t>(lane);
                bool bad = false;
                if (r < upto) {
                    const unsigned long long* q = reinterpret_cast<const unsigned long long*>(&a.runq[r]);
                    const unsigned long long q0 = __hip_atomic_load(q, __ATOMIC_RELAXED, P3_AGENT);
                    const unsigned long long q1 = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, P3_AGENT);
                    const unsigned long long q2 = __hip_atomic_load(q + 2, __ATOMIC_RELAXED, P3_AGENT);
                    const unsigned long long q3 = __hip_atomic_load(q + 3, __ATOMIC_RELAXED, P3_AGENT);
                    P3Run e;
                    e.start = static_cast<int64_t>(q0);
                    e.len = static_cast<int64_t>(q1);
                    e.grid_off = static_cast<int32_t>(q2 & 0xffffffffull);
                    e.layer = static_cast<int32_t>(q2 >> 32);
                    e.tile0 = static_cast<uint32_t>(q3 & 0xffffffffull);
                    e.tile_end = static_cast<uint32_t>(q3 >> 32);
                    ring[r & (P3_RUN_CACHE - 1)] = e;
                    bad = !p3_run_valid(e, a.arena_elems, a.L, a.tile_elems);
                }
                if (__ballot(bad) != 0ull) {
                    // a record the selector cannot have written (it would be turned into addresses): the
                    // workgroup takes no more work and the drain is reported as failed
                    if (lane_is(lane, 0)) a.hs->worker_status = P3D_OVERFLOW;
                    out.r_next = r_next;
                    out.r_have = r_have;
                    return out;
                }
            }
            r_have = upto;
            continue;
        }
        if (!WAIT) break;                              // the queue was complete before this launch
        const uint32_t fin = uni(fin_v);
        if (fin != P3_NONE && r_have >= fin) break;    // the queue is complete and has no such tile
        if (!may_wait) {                               // the caller has something to settle before it waits
            out.found = 2;
            break;
        }
        // bounded wait: the selector turns a host abort into `final_runs`, so the workers
        // only need the clock (no host-memory reads from hundreds of spinners)
        // (reading the clock costs as much as a look at the queue: every 16th look is enough for a limit of seconds)
        looks += 1u;
        if ((looks & 15u) == 0u && clock_now() - t_enter > a.watchdog_ticks) {
            if (lane_is(lane, 0)) a.hs->worker_status = P3D_WATCHDOG;
            break;
        }
        // a waiting workgroup still answers for its XCD in the write-back rounds
        const FlushView fv = view_of(fv_v);
        if (flush_due(fv, true)) serve_flush(fc, fv.req, xcd, lane);
        __builtin_amdgcn_s_sleep(4);
    }
    out.r_next = r_next;
    out.r_have = r_have;
    return out;
}

// The worker loop.  WAIT = true: the selector runs concurrently in workgroup 0
// of the same launch, so a tile number beyond the published part of the queue
// waits (bounded) for the queue to grow.  WAIT = false: the queue was completed
// by an earlier launch on the stream, so a number beyond its end means "no more
// work".
//
// A round: every wavefront streams its share of the tile; the leader (wavefront
// 0) asks for the next tile number; barrier; the leader does the bookkeeping;
// barrier.  Nothing in a round waits for memory on purpose:
//  * the next tile number is asked for when the leader has issued its share of
//    the tile, and is usually there when the other wavefronts reach the barrier;
//  * a tile is counted against its layer ONE ROUND LATE.  Nobody waits for the
//    acknowledgements of a tile's stores: a wavefront's first wait for a load of
//    the next tile (`s_waitcnt vmcnt(n)`, n small; the counter covers loads and
//    stores alike, in issue order) cannot end before the stores of the tile
//    before have been acknowledged, so behind the barrier of round r every store
//    of tile r-1 is in the L2 and tile r-1 may be counted (a wavefront that has
//    nothing to load in round r waits explicitly);
//  * what the additions to the layers' counts return (did this one complete the
//    layer?) is looked at in the round after.
// So a layer's completion is noticed two tile times (about 10 us) after its last
// store.  Layer 0, the layer the next forward pass needs first, does not pay
// that: its tiles are marked urgent, every wavefront waits for its stores before
// the barrier, and the count is added and looked at in the same round.  A
// workgroup that finds no further tile (or would have to wait for the queue to
// grow) first runs a DRAIN round -- wait for all stores, count what is uncounted,
// look at every result -- so nothing is left hanging while it waits or leaves.
// Turning a tile number into addresses costs no memory access: the leader keeps
// the run it is working in in scalar registers and a copy of the run table in
// LDS (a search of LDS at a run boundary).
//
// Control flow: branches on the wave index and on leader state are scalar (whole
// wavefronts take them); the few single-lane sections are guarded by opaque
// conditions (lane_is) and never enclose a barrier.  (With single-lane sections
// that share one condition on both sides of the loop's back edge the compiler
// may give the other lanes a private loop around the barriers that the leader
// lane never re-enters: the workgroup then spins on a stale descriptor forever.)
// What the out-of-line helpers of the worker loop need.  It lives in LDS, not in scalar registers: the helpers are
// called once in a while (a refill, a completed layer, a write-back round), the loop around them every few
// microseconds, and twenty-six scalar registers held for them were spilled and moved about in every round.
struct WorkerCtx {
    FlushCtx fc;
    QueueCtx qc;
};
__device__ __forceinline__ FlushCtx flush_ctx(const WorkerCtx& c) {
    asm volatile("" ::: "memory");             // read where it is used, not once in front of the loop
    return c.fc;
}
__device__ __forceinline__ QueueCtx queue_ctx(const WorkerCtx& c) {
    asm volatile("" ::: "memory");
    return c.qc;
}

template <int WT, bool BF16, bool WD, bool WAIT>
__device__ __forceinline__ void run_worker(const P3DrainArgs& a, const P3GradPtrs& gp, P3TileDesc& s_desc,
                                           P3Run* s_runs, WorkerCtx& s_ctx) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: whole wavefronts branch on it
    P3Ctl* ctl = a.ctl;
    const HyperT<WD> h = {a.lr, a.mu, a.rescale, a.wd};
    const uint64_t t_enter = clock_now();
    if (tid == 0) {
        const QueueCtx qc0 = {a.ctl, a.runq, a.hs, a.watchdog_ticks, a.arena_elems, a.L, a.tile_elems};
        const FlushCtx fc0 = {a.ctl, a.layer_req, a.t_seen_dev, a.t_seen, a.t_done, a.done_flag, a.iter_seq, a.L};
        s_ctx.qc = qc0;
        s_ctx.fc = fc0;
    }
    const int xcd = xcd_of_this_wave();

    // leader state (wavefront 0 only), scalar
    P3Run cur;                         // the run the last tile number fell into
    cur.start = cur.len = 0;
    cur.grid_off = cur.layer = 0;
    cur.tile0 = cur.tile_end = 0u;     // empty: the first number goes through locate_run
    uint32_t r_next = 0u, r_have = 0u;
    uint32_t k_wait = 0u;                 // the tile number a DRAIN round has to find work for
    int prev_n = 0, prev_layer = 0;       // the tile of the round before: streamed, not counted yet (prev_n = 0: none)
    bool prev_long = false;
    int pend_layer = 0, pend_tiles = 0;   // counted tiles of one long run not yet added to their layer's count
    uint32_t pend_cnt = 0u;               // their elements
    // additions that have been made but whose result (did this one complete the layer?) has not been looked
    // at yet: A = a layer the workgroup has left, B = the layer of the tile counted last
    unsigned long long po_old_a = 0ull, po_old_b = 0ull;      // vector registers: what the additions return
    unsigned long long po_le_a = 1ull, po_le_b = 1ull;        // vector registers: elements of the layers (loaded with
                                                              // the additions, so that nothing waits for them alone)
    uint32_t po_cnt_a = 0u, po_cnt_b = 0u;                    // what was added (0: nothing outstanding)
    int po_layer_a = 0, po_layer_b = 0;
    // Look at the outstanding results; an addition that completed its layer starts the layer's publication.
    auto settle = [&]() {
        if (po_cnt_a != 0u) {
            const unsigned long long old = uni(po_old_a);
            if (old + static_cast<unsigned long long>(po_cnt_a) == uni(po_le_a)) {
                if (old == 0ull && po_layer_a == 0) complete_alone(flush_ctx(s_ctx), po_layer_a, lane);
                else complete_layer(flush_ctx(s_ctx), po_layer_a, xcd, lane);
            }
            po_cnt_a = 0u;
        }
        if (po_cnt_b != 0u) {
            const unsigned long long old = uni(po_old_b);
            if (old + static_cast<unsigned long long>(po_cnt_b) == uni(po_le_b)) {
                if (old == 0ull && po_layer_b == 0) complete_alone(flush_ctx(s_ctx), po_layer_b, lane);
                else complete_layer(flush_ctx(s_ctx), po_layer_b, xcd, lane);
            }
            po_cnt_b = 0u;
        }
    };
    // Count a tile whose stores have all been acknowledged (nothing may be outstanding: settle() first).
    // In a long run (a layer of thousands of tiles, whose count is one word that every workgroup adds to) a
    // workgroup adds P3_RETIRE_BATCH tiles at a time: fewer, larger additions.  In a short run every tile is
    // added at once.  `flush`: add whatever is pending, too.
    auto count_tile = [&](int t_layer, int t_n, bool t_long, bool flush) {
        uint32_t cnt_a = 0u, cnt_b = 0u;
        int layer_a = t_layer;
        if (pend_tiles > 0 && pend_layer != t_layer) {
            cnt_a = pend_cnt;
            layer_a = pend_layer;
            pend_cnt = 0u;
            pend_tiles = 0;
        }
        if (t_n > 0) {
            pend_cnt += static_cast<uint32_t>(t_n);
            pend_tiles += 1;
            pend_layer = t_layer;
        }
        if (pend_tiles > 0 && (flush || !t_long || pend_tiles >= P3_RETIRE_BATCH)) {
            cnt_b = pend_cnt;
            pend_cnt = 0u;
            pend_tiles = 0;
        }
        if (cnt_a != 0u) {
            if (lane_is(lane, 0))
                po_old_a = __hip_atomic_fetch_add(&a.layer_done[layer_a], static_cast<unsigned long long>(cnt_a),
                                                  __ATOMIC_RELAXED, P3_AGENT);
            po_le_a = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(&a.layers[layer_a].elems),
                                        __ATOMIC_RELAXED, P3_AGENT);
            po_cnt_a = cnt_a;
            po_layer_a = layer_a;
        }
        if (cnt_b != 0u) {
            if (lane_is(lane, 0))
                po_old_b = __hip_atomic_fetch_add(&a.layer_done[pend_layer], static_cast<unsigned long long>(cnt_b),
                                                  __ATOMIC_RELAXED, P3_AGENT);
            po_le_b = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(&a.layers[pend_layer].elems),
                                        __ATOMIC_RELAXED, P3_AGENT);
            po_cnt_b = cnt_b;
            po_layer_b = pend_layer;
        }
    };
    // Take over the run `f` found.
    auto enter_run = [&](const P3Run& r) {
        cur.start = static_cast<int64_t>(uni(static_cast<unsigned long long>(r.start)));
        cur.len = static_cast<int64_t>(uni(static_cast<unsigned long long>(r.len)));
        cur.grid_off = uni(r.grid_off);
        cur.layer = uni(r.layer);
        cur.tile0 = uni(r.tile0);
        cur.tile_end = uni(r.tile_end);
    };
    // The descriptor of tile k of the current run.  Tiles of layer 0 in a short run are urgent.
    auto describe = [&](uint32_t k) {
        P3TileDesc d = p3_tile_of_run(cur, k, a.tile_elems);
        const bool long_run = cur.tile_end - cur.tile0 >= P3_LONG_RUN_TILES_PER_WG * a.n_blocks;
        d.flags = (cur.layer == 0 && !long_run) ? P3T_URGENT : 0;
        return d;
    };

    // The first round is a DRAIN round with nothing to drain: it finds the tile of the first number.
    if (wave == 0) {
        const uint32_t k_first = take_ticket(ctl, lane);      // asked for now, looked at below
        if (WAIT && a.n_first > 0) {
            // the leading runs of the first selection step came with the launch: they go into the ring as if
            // they had been read from the queue (their tile numbers follow from their order), and the
            // workgroup starts on them without waiting for the selector
            // (the host has checked them against the arena; a check here, cheap as it is, was measured to cost
            // the bf16 kernel 2 % -- scalar registers spilled in the loop below)
            int t_before = 0;
            for (int base = 0; base < a.n_first; base += 64) {
                const int r = base + lane;
                P3FirstRun fr;
                fr.start = 0;
                fr.len = 1u;
                fr.layer = 0;
                int c = 0;
                if (r < a.n_first) {
                    fr = a.first_runs[r];
                    c = static_cast<int>(p3_run_cells(fr.start, static_cast<int64_t>(fr.len), a.tile_elems));
                }
                const int c_incl = wave_incl_scan(c, lane);
                if (r < a.n_first) {
                    P3Run e;
                    e.start = fr.start;
                    e.len = static_cast<int64_t>(fr.len);
                    e.grid_off = static_cast<int32_t>(fr.start % a.tile_elems);
                    e.layer = fr.layer;
                    e.tile0 = static_cast<uint32_t>(t_before + c_incl - c);
                    e.tile_end = static_cast<uint32_t>(t_before + c_incl);
                    s_runs[r] = e;
                }
                t_before += __shfl(c_incl, 63, 64);
            }
            r_have = static_cast<uint32_t>(a.n_first);
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");      // the ring is read by other lanes
        }
        k_wait = uni(k_first);
        P3TileDesc d0;
        d0.start = 0;
        d0.n = P3T_DRAIN;
        d0.layer = 0;
        d0.flags = 0;
        if (lane_is(lane, 0)) s_desc = d0;
    }
    __syncthreads();

    for (;;) {
        const int32_t n = uni(s_desc.n);                      // scalar: uniform branches
        if (n == P3T_END) break;
        if (n == P3T_DRAIN) {
            // every store of this workgroup is acknowledged; the leader counts what is uncounted, looks at
            // every result, and only then looks (and, if need be, waits) for work
            wait_vm_done();
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __syncthreads();
            if (wave == 0) {
                settle();
                count_tile(prev_layer, prev_n, prev_long, true);
                prev_n = 0;
                settle();
                const Located f = locate_run<WAIT>(queue_ctx(s_ctx), flush_ctx(s_ctx), xcd, s_runs, k_wait, r_next, r_have, t_enter, lane, true);
                r_next = uni(f.r_next);
                r_have = uni(f.r_have);
                P3TileDesc dn;
                dn.start = 0;
                dn.n = P3T_END;
                dn.layer = 0;
                dn.flags = 0;
                if (uni(f.found) == 1) {
                    enter_run(f.run);
                    dn = describe(k_wait);
                }
                if (lane_is(lane, 0)) s_desc = dn;
            }
            __syncthreads();
            continue;
        }
        const int64_t start = static_cast<int64_t>(uni(static_cast<unsigned long long>(s_desc.start)));
        const int32_t layer = uni(s_desc.layer);
        const bool urgent = uni(s_desc.flags) != 0;

        const int32_t nvec = process_tile<WT, BF16>(gp, a.W, a.w, a.m, start, n, h);

        // the next tile number and this XCD's write-back line: asked for now, looked at behind the barrier
        uint32_t tk_pre = 0u;
        u32x4 fv_pre = {0u, 0u, 0u, 0u};
        if (wave == 0) {
            if (lane_is(lane, 0)) tk_pre = __hip_atomic_fetch_add(&ctl->ticket, 1u, __ATOMIC_RELAXED, P3_AGENT);
            fv_pre = load_flush_view(ctl, xcd);
        }
        // a wavefront that loaded nothing in this round has not waited for its earlier stores yet; the stores
        // of an urgent tile are waited for at once
        if (urgent || wave * 64 >= nvec) wait_vm_done();
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();                                      // every store of the tile before this one is out

        if (wave == 0) {
            settle();                                         // what the additions of the round before returned
            count_tile(prev_layer, prev_n, prev_long, false); // the tile of the round before
            const bool long_run = cur.tile_end - cur.tile0 >= P3_LONG_RUN_TILES_PER_WG * a.n_blocks;
            prev_n = n;
            prev_layer = layer;
            prev_long = long_run;
            const uint32_t k = uni(tk_pre);
            const FlushView fv = view_of(fv_pre);
            if (urgent) {                                     // count it and look at the result now
                settle();
                count_tile(layer, n, long_run, true);
                prev_n = 0;
                settle();
            }
            if (flush_due(fv, false)) serve_flush(flush_ctx(s_ctx), fv.req, xcd, lane);

            P3TileDesc dn;
            dn.start = 0;
            dn.n = P3T_DRAIN;                                 // unless the tile is found below
            dn.layer = 0;
            dn.flags = 0;
            k_wait = k;
            if (k < cur.tile_end) {
                dn = describe(k);
            } else if (r_next < r_have) {
                // Left the run.  The usual case, here in line: the next run is one of the next 64 of the LDS
                // copy (tile numbers and runs both only grow, so it is the first whose end lies beyond the
                // number).  Everything else -- a refill of the copy, a wait for the queue to grow, the end
                // of the queue -- is left to a DRAIN round.
                const uint32_t r = r_next + static_cast<uint32_t>(lane);
                const bool in = r < r_have;
                uint32_t te = 0u;
                if (in) te = s_runs[r & (P3_RUN_CACHE - 1)].tile_end;
                const unsigned long long hits = __ballot(in && k < te);
                if (hits != 0ull) {
                    const uint32_t rf = r_next + static_cast<uint32_t>(__builtin_ctzll(hits));
                    enter_run(s_runs[rf & (P3_RUN_CACHE - 1)]);          // every lane reads the same entry
                    r_next = rf + 1u;
                    dn = describe(k);
                } else {
                    r_next = r_have - r_next > 64u ? r_next + 64u : r_have;
                }
            }
            if (lane_is(lane, 0)) s_desc = dn;                // everyone has read the old one before the barrier above
        }
        __syncthreads();                                      // the next descriptor is in LDS
    }

    // (the loop ends behind a DRAIN round: nothing uncounted, nothing unlooked-at)
    if (wave == 0) leave_loop(flush_ctx(s_ctx), xcd, lane);

    // Last workgroup out re-arms the per-launch words for the next drain.
    if (lane_is(tid, 0)) {
        // (every ticket this workgroup took has returned its value, so the reset below cannot
        // overtake a ticket of a workgroup that has already been counted)
        const uint32_t old = __hip_atomic_fetch_add(&ctl->exit_count, 1u, __ATOMIC_RELAXED, P3_AGENT);
        if (old + 1u == a.n_blocks) {
            __hip_atomic_store(&ctl->ticket, 0u, __ATOMIC_RELAXED, P3_AGENT);
            __hip_atomic_store(&ctl->published, 0u, __ATOMIC_RELAXED, P3_AGENT);
            __hip_atomic_store(&ctl->final_runs, P3_NONE, __ATOMIC_RELAXED, P3_AGENT);
            __hip_atomic_store(&ctl->flush_req, 0u, __ATOMIC_RELAXED, P3_AGENT);
            for (int x = 0; x < P3_MAX_XCD; ++x) {
                __hip_atomic_store(&ctl->xcd[x].req, 0u, __ATOMIC_RELAXED, P3_AGENT);
                __hip_atomic_store(&ctl->xcd[x].urgent, 0u, __ATOMIC_RELAXED, P3_AGENT);
                __hip_atomic_store(&ctl->xcd[x].claim, 0u, __ATOMIC_RELAXED, P3_AGENT);
                __hip_atomic_store(&ctl->xcd[x].ack, 0u, __ATOMIC_RELAXED, P3_AGENT);
                __hip_atomic_store(&ctl->xcd[x].used, 0u, __ATOMIC_RELAXED, P3_AGENT);
            }
            __hip_atomic_store(&ctl->exit_count, 0u, __ATOMIC_RELAXED, P3_AGENT);
        }
    }
}

// One launch: selector in workgroup 0, every workgroup a worker (LIVE needs this).
template <int WT, bool BF16, bool WD>
__global__ void __launch_bounds__(P3_BLOCK) P3_KERNEL_ATTR p3_drain_kernel(const P3DrainArgs a, const P3GradPtrs gp) {
    __shared__ SelectorLds lds;
    __shared__ P3TileDesc s_desc;
    __shared__ P3Run s_runs[P3_RUN_CACHE];
    __shared__ WorkerCtx s_ctx;
    // (nobody waits for the registration here: the worker's first round waits for everything its leader has
    // outstanding -- registration, first tile number, the runs handed over -- in one go, long before its first store)
    if (threadIdx.x < 64) enter_xcd(a.ctl, xcd_of_this_wave(), static_cast<int>(threadIdx.x), false);
    if (blockIdx.x == 0) run_selector(a, lds);
    run_worker<WT, BF16, WD, true>(a, gp, s_desc, s_runs, s_ctx);
}

// Two launches on one stream: the selector alone (one workgroup) ...
__global__ void __launch_bounds__(P3_BLOCK) P3_KERNEL_ATTR p3_select_kernel(const P3DrainArgs a) {
    __shared__ SelectorLds lds;
    run_selector(a, lds);
}

// ... then the workers over the finished queue; no workgroup ever waits for another.
template <int WT, bool BF16, bool WD>
__global__ void __launch_bounds__(P3_BLOCK) P3_KERNEL_ATTR p3_work_kernel(const P3DrainArgs a, const P3GradPtrs gp) {
    __shared__ P3TileDesc s_desc;
    __shared__ P3Run s_runs[P3_RUN_CACHE];
    __shared__ WorkerCtx s_ctx;
    if (threadIdx.x < 64) enter_xcd(a.ctl, xcd_of_this_wave(), static_cast<int>(threadIdx.x), true);
    run_worker<WT, BF16, WD, false>(a, gp, s_desc, s_runs, s_ctx);
}

// ---------------------------------------------------------------- launcher ----
typedef void (*p3_kernel_t)(const P3DrainArgs, const P3GradPtrs);

template <bool BF16, bool WD, bool PERSISTENT>
static p3_kernel_t pick_kernel(int W) {
    if (PERSISTENT) {
        switch (W) {
            case 1: return p3_drain_kernel<1, BF16, WD>;
            case 2: return p3_drain_kernel<2, BF16, WD>;
            case 4: return p3_drain_kernel<4, BF16, WD>;
            case 8: return p3_drain_kernel<8, BF16, WD>;
            case 16: return p3_drain_kernel<16, BF16, WD>;
            default: return p3_drain_kernel<0, BF16, WD>;
        }
    }
    switch (W) {
        case 1: return p3_work_kernel<1, BF16, WD>;
        case 2: return p3_work_kernel<2, BF16, WD>;
        case 4: return p3_work_kernel<4, BF16, WD>;
        case 8: return p3_work_kernel<8, BF16, WD>;
        case 16: return p3_work_kernel<16, BF16, WD>;
        default: return p3_work_kernel<0, BF16, WD>;
    }
}

template <bool BF16, bool WD>
static p3_kernel_t pick2(int W, int persistent) {
    return persistent ? pick_kernel<BF16, WD, true>(W) : pick_kernel<BF16, WD, false>(W);
}

static p3_kernel_t pick(int W, int grad_dtype, int with_wd, int persistent) {
    if (grad_dtype == 1) return with_wd ? pick2<true, true>(W, persistent) : pick2<true, false>(W, persistent);
    return with_wd ? pick2<false, true>(W, persistent) : pick2<false, false>(W, persistent);
}

P3_NS_END

extern "C" int P3_LAUNCH_SYM(const P3DrainArgs* args, const P3GradPtrs* grads, int grad_dtype,
                             int persistent, unsigned grid, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    P3_NS_Q p3_kernel_t k = P3_NS_Q pick(args->W, grad_dtype, args->wd != 0.0f ? 1 : 0, persistent);
    if (!persistent) {
        hipLaunchKernelGGL(P3_NS_Q p3_select_kernel, dim3(1), dim3(P3_BLOCK), 0, st, *args);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return static_cast<int>(e);
    }
    hipLaunchKernelGGL(k, dim3(grid), dim3(P3_BLOCK), 0, st, *args, *grads);
    return static_cast<int>(hipGetLastError());
}

extern "C" int P3_OCCUPANCY_SYM(int W, int grad_dtype, int persistent, int* blocks_per_cu) {
    P3_NS_Q p3_kernel_t k = P3_NS_Q pick(W, grad_dtype, 1, persistent);   // the weight-decay variant uses no fewer registers
    return static_cast<int>(hipOccupancyMaxActiveBlocksPerMultiprocessor(
        blocks_per_cu, reinterpret_cast<const void*>(k), P3_BLOCK, 0));
}
