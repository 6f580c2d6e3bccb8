// Internal structures shared by the host runtime and the gfx950 drain kernel.
// Not part of the public ABI (that is include/p3.h).
#ifndef P3_INTERNAL_H_
#define P3_INTERNAL_H_

#include <stdint.h>

#include "p3_tiles.h"

// The drain kernel is built twice from one source.  The wide build is the default: one workgroup owns a
// compute unit.  The lean build (p3_drain_lean.hip) has workgroups of four wavefronts with at most 128
// registers a lane, a quarter of each SIMD's register file, so that workgroups of other kernels -- a backward
// pass on another stream -- find room on the same compute unit while the drain is resident.
#ifndef P3_BLOCK
#define P3_BLOCK 832            // threads per workgroup = 13 wavefronts of 64, one workgroup per CU (measured optimum
                                // with the arenas well placed: 704 lanes 1.067 ms, 768 1.032, 832 1.020, 896 1.035, 960 1.045)
#endif
#define P3_BLOCK_LEAN 256       // threads per workgroup of the lean build
#define P3_TILE_LEAN 4096       // its default tile: four steps of the workgroup
#define P3_WAVES (P3_BLOCK / 64)
#define P3_BATCH_MAX P3_BLOCK   // slices the selector claims per publication step (one per selector thread)
#define P3_NONE 0xffffffffu     // "final queue length not known yet"
#define P3_MAXW 64
#define P3_MAX_XCD 16           // L2 caches (accelerator complex dies) a launch can be spread over
#define P3_RETIRE_BATCH 4           // tiles of one long run a workgroup finishes before it adds them to the layer's count
#define P3_LONG_RUN_TILES_PER_WG 8u // a run is long when it gives every workgroup at least this many tiles
#define P3_PUBLISHED 0x80000000u   // layer_req: the layer's done flag has been written
#define P3_FLUSH_GAP_TICKS 5000u   // busy workgroups leave 50 us (100 MHz clock) between two write-backs of one L2 ...
#define P3_URGENT_LAYERS 8         // ... except for the completion of one of the first layers (the forward pass is waiting)
#define P3_INLINE_MARKS 256      // marks handed to a SNAPSHOT/TICKED drain with its launch arguments
#define P3_INLINE_RUNS 128       // runs of the first selection step handed to a SNAPSHOT drain with its launch arguments

// Device-side status of a drain (written to pinned host memory at its end).
enum { P3D_OK = 0, P3D_WATCHDOG = 1, P3D_ABORTED = 2, P3D_OVERFLOW = 3 };

// layer_state values (device)
enum { P3L_IDLE = 0, P3L_PENDING = 1, P3L_RELEASED = 2 };

// A run of the first selection step as the host hands it over: its tile numbers follow from the order.
struct P3FirstRun {
    int64_t start;
    uint32_t len;
    int32_t layer;
};

// One slice: a contiguous run of one layer (Sec. 4.2).  start is an element
// offset into every arena.  32 bytes, so the selector needs one load per slice.
struct P3SliceDev {
    int64_t start;
    int32_t len;
    int32_t layer;
    int32_t layer_slices;   // slices of the parent layer
    int32_t index_in_layer; // 0 for the layer's first slice; slice g-1 precedes slice g in memory when > 0
    int64_t layer_elems;    // parameters of the parent layer
};

struct P3LayerDev {
    int32_t first;   // first global slice id
    int32_t count;   // number of slices
    int64_t elems;   // parameters of the layer
};

#ifndef P3_RUN_CACHE
#define P3_RUN_CACHE 512    // run records a workgroup keeps in LDS (a ring; power of two)
#endif
#ifndef P3_LDS_BM_WORDS
#define P3_LDS_BM_WORDS 4096   // the selector keeps the ready bitmap in LDS when it has at most this many words (262,144 slices)
#endif
#define P3_LDS_LAYERS 2048     // ... and the layer states when there are at most this many layers

// Per-XCD part of the write-back rounds.  Every leader reads the first 16 bytes of
// its XCD's line once per tile (one 128-bit load); keeping them per XCD spreads that
// traffic over as many memory channels (control words that all 256 workgroups read
// uncached every tile load one channel enough to slow the whole stream: measured).
struct alignas(128) P3XcdCtl {
    uint32_t req;      // highest round this XCD has been told of (written by the workgroup that opened it)
    uint32_t urgent;   // highest round of layer 0 it has been told of
    uint32_t claim;    // highest round one of its workgroups has undertaken to write back for
    uint32_t time32;   // device clock (low 32 bits) when its last write-back began
    uint32_t ack;      // highest round whose write-back is complete
    uint32_t live;     // workgroups of this launch that have not left yet
    uint32_t used;     // this launch has (had) workgroups here
    uint32_t pad;
};

// Device control block.  Hot words sit on their own 128-byte lines.
struct P3Ctl {
    // per launch; reset by the last workgroup to leave the kernel
    alignas(128) uint32_t ticket;       // tiles handed out so far
    alignas(128) uint32_t published;    // runs present in the queue
    alignas(128) uint32_t final_runs;   // P3_NONE until the selector has finished; then the length of the queue
    alignas(128) uint32_t exit_count;
    // write-back rounds (see the worker loop): per launch, re-armed like the words above
    alignas(128) uint32_t flush_req;    // layers completed so far = write-back rounds opened
    P3XcdCtl xcd[P3_MAX_XCD];           // one 128-byte line per XCD
    // selector state; lives across the drains of one iteration
    alignas(128) uint32_t claimed;      // slices claimed so far this iteration
    uint32_t marks_applied;             // marks of this iteration already folded into the bitmap
    uint32_t n_ready;                   // ready, unclaimed slices
    uint32_t lo_word;                   // no set bit below this bitmap word
    uint32_t pending;                   // TICKED: layers marked but not yet released
    uint32_t pad0;
    int64_t clock;                      // TICKED: logical tick
    // first-come-first-served policy: layers are served whole, in the order they became ready
    uint32_t fifo_head, fifo_tail;      // arrival queue (SNAPSHOT/LIVE): served / appended so far
    uint32_t cur_next, cur_left;        // next slice of the layer being served, and how many of its slices are left
};

// Pinned host memory the kernel reads (marks, abort) and writes (flags, stamps).
struct P3HostShared {
    alignas(64) uint64_t n_marks;       // absolute number of marks ever issued (host -> device)
    alignas(64) uint32_t abort_flag;    // host -> device
    alignas(64) uint32_t last_claimed;  // device -> host at the end of a drain
    uint32_t last_status;
    uint32_t last_iter;
    alignas(64) uint32_t phase;         // device -> host: selector progress of the running drain (diagnostics)
    uint32_t worker_status;             // device -> host: set by a worker that gave up waiting
    alignas(64) uint64_t t_sel_enter;   // device clock: selector entered / first queue growth / selection finished
    uint64_t t_sel_first_pub;
    uint64_t t_sel_final;
};

// selector progress codes written to P3HostShared::phase
enum { P3P_PUBLISHED = 5, P3P_FINAL = 6 };

struct P3GradPtrs {
    const void* p[P3_MAXW];
};

// Everything one drain launch needs, passed by value.
struct P3DrainArgs {
    // tables (device)
    const P3SliceDev* slices;
    const P3LayerDev* layers;
    const int64_t* release;       // TICKED: release tick per layer
    unsigned long long* bitmap;   // ready & unclaimed, one bit per slice
    uint8_t* layer_state;
    P3Run* runq;
    int32_t* order;               // claim log
    int32_t* epoch;               // marks observed at each claim
    unsigned long long* layer_done;   // elements retired per layer this iteration
    uint32_t* layer_req;          // per layer: 0, or the write-back round its completion asked for (| P3_PUBLISHED)
    // The two arrays above exist twice and iterations alternate between the sets: the first drain of an
    // iteration clears the set the NEXT iteration will use (nobody else touches it meanwhile), so the set in
    // use is clean before the launch and a worker may count a tile as early as it likes.  NULL: nothing to clear.
    unsigned long long* layer_done_next;
    uint32_t* layer_req_next;
    int32_t* fifo;                // first-come-first-served policy: layers in the order they became ready
    uint64_t* t_seen_dev;         // per layer: device clock when the selector saw it ready
    P3Ctl* ctl;
    // pinned host memory
    P3HostShared* hs;
    const unsigned long long* mark_log;   // ring of marks in mark order: (low 32 bits of absolute index + 1) << 32 | layer
    uint32_t* done_flag;          // per layer: iteration number once complete
    uint64_t* t_seen;             // per layer: copy of t_seen_dev, written when the layer completes
    uint64_t* t_done;             // per layer: device clock when its last tile retired
    // data (device)
    float* w;
    float* m;
    // sizes
    int64_t arena_elems;          // elements of every arena: no run may reach beyond
    int32_t K;
    int32_t L;
    int32_t n_words;
    uint32_t mark_cap;
    uint32_t run_cap;             // entries in runq
    int32_t tile_elems;
    int32_t tiles_per_full_slice;
    // this launch
    uint64_t epoch_base;          // absolute index of this iteration's first mark
    uint64_t epoch_limit;         // SNAPSHOT/TICKED: marks issued before the drain call
    uint64_t watchdog_ticks;      // every wait in the kernel gives up after this many device clock ticks
    uint32_t lookahead;           // LIVE: tiles the selector may run ahead
    uint32_t iter_seq;
    int32_t mode;
    int32_t policy;               // 0: most urgent ready slice first (P3); 1: layers whole, first come first served
    int32_t iter_begin;           // first drain of the iteration: clear per-iteration state
    uint32_t n_blocks;
    int32_t W;
    float lr, mu, rescale, wd;
    // SNAPSHOT/TICKED: the marks this drain has to fold, in mark order, when they fit
    // (else n_inline = 0 and the kernel reads the pinned mark log over the host link)
    int32_t n_inline;
    int32_t inline_marks[P3_INLINE_MARKS];
    // A drain in SNAPSHOT mode under the priority rule: what the selector's first step will claim follows
    // from the drain's marks alone, so the host works its leading runs out (p3_first_step_runs)
    // and hands them over with the launch.  Every workgroup starts on them at once instead of waiting 10 us for
    // the first publication; the selector produces the same records in its first step, checks them against
    // these, and ends the drain with an error if one differs.  That first step is a full one then (P3_BATCH_MAX
    // slices: nobody is waiting for it, and the runs handed over should last until it is published).  0: none.
    int32_t n_first;
    P3FirstRun first_runs[P3_INLINE_RUNS];
};

#ifdef __cplusplus
extern "C" {
#endif
// Defined in p3_drain.hip.  stream is a hipStream_t.  Returns a hipError_t as int.
// persistent != 0: one launch (selector + workers); 0: selector launch, then worker launch.
int p3_launch_drain(const P3DrainArgs* args, const P3GradPtrs* grads, int grad_dtype,
                    int persistent, unsigned grid, void* stream);
// Resident workgroups per compute unit of the kernel that (W, dtype, persistent) selects.
int p3_drain_occupancy(int W, int grad_dtype, int persistent, int* blocks_per_cu);
// The same two for the lean build (defined in p3_drain_lean.hip).
int p3_launch_drain_lean(const P3DrainArgs* args, const P3GradPtrs* grads, int grad_dtype,
                         int persistent, unsigned grid, void* stream);
int p3_drain_occupancy_lean(int W, int grad_dtype, int persistent, int* blocks_per_cu);
#ifdef __cplusplus
}
#endif

#endif  // P3_INTERNAL_H_
