// Runs and tiles: how a claimed stretch of the arenas is cut into the units one
// workgroup streams (Sec. 4.2: a slice that has been taken is finished, and
// nothing outside it is touched).  Plain integer arithmetic with no device
// intrinsics, so the same code is compiled into the gfx950 kernel and, for the
// host-side arithmetic tests, by an ordinary C++ compiler.
#ifndef P3_TILES_H_
#define P3_TILES_H_

#include <stdint.h>

#if defined(__HIPCC__)
#define P3_HD __host__ __device__ __forceinline__
#else
#define P3_HD inline
#endif

// The work queue holds RUNS.  Slices that were claimed in one selection step,
// belong to one layer and follow each other in memory form a run; the claim
// order is the order of the runs and, inside a run, of the addresses.  A run is
// processed as tiles: the cells of a grid of tile_elems elements laid over the
// arena, clipped to the run (so a tile may span the boundary of two slices of the
// run -- neighbours in the claim order -- and every tile but a run's first starts
// on a multiple of tile_elems).  Tiles are numbered through the whole queue;
// a worker draws a tile number and finds its run in a copy of the run table
// that its workgroup keeps in LDS, so a tile costs no queue access at all.
struct P3Run {
    int64_t start;        // element offset into the arenas
    int64_t len;          // elements
    int32_t grid_off;     // start - (start / tile_elems) * tile_elems
    int32_t layer;        // owning layer
    uint32_t tile0;       // number of the run's first tile
    uint32_t tile_end;    // tile0 + tiles of the run
};

// What a workgroup works on in one round (LDS only).
struct P3TileDesc {
    int64_t start;        // element offset into the arenas
    int32_t n;            // elements, or P3T_END / P3T_DRAIN
    int32_t layer;        // owning layer
    int32_t flags;        // P3T_URGENT or 0
    int32_t pad;
};
enum { P3T_END = -1, P3T_DRAIN = -2 };   // no more work / a round without a tile (see the worker loop)
enum { P3T_URGENT = 1 };                 // the tile's completion is counted in its own round

// Grid cells (= tiles) that the stretch [start, start+len) touches; len >= 1.
P3_HD int64_t p3_run_cells(int64_t start, int64_t len, int32_t tile_elems) {
    return (start + len - 1) / tile_elems - start / tile_elems + 1;
}

// How many slices the first selection step of a launch claims at most: enough to give every workgroup two
// tiles, at least what one wavefront groups on its own, at most 256.  (The host works the first step of a
// snapshot drain out ahead of the launch with the same rule; see P3FirstRun.)
P3_HD int32_t p3_first_step_slices(uint32_t n_blocks, int32_t tiles_per_full_slice) {
    int32_t cap = (2 * static_cast<int32_t>(n_blocks) + tiles_per_full_slice - 1) / tiles_per_full_slice;
    return cap < 64 ? 64 : (cap > 256 ? 256 : cap);
}

// Is this record one the selector can have written for an arena of arena_elems elements and L layers?
// Every address a worker derives from a record that passes lies inside [start, start+len), and that
// inside the arena -- so a record read stale or torn ends the drain with an error instead of becoming
// a wild address.
P3_HD bool p3_run_valid(const P3Run& r, int64_t arena_elems, int32_t n_layers, int32_t tile_elems) {
    if (r.start < 0 || r.len < 1 || r.start > arena_elems || r.len > arena_elems - r.start) return false;
    if (r.layer < 0 || r.layer >= n_layers) return false;
    if (r.grid_off < 0 || static_cast<int64_t>(r.grid_off) != r.start % tile_elems) return false;
    if (r.tile_end <= r.tile0) return false;
    return static_cast<int64_t>(r.tile_end - r.tile0) == p3_run_cells(r.start, r.len, tile_elems);
}

// Tile k of the queue, given the run that holds it (tile0 <= k < tile_end): grid cell (k - tile0) of the run, clipped.
P3_HD P3TileDesc p3_tile_of_run(const P3Run& r, uint32_t k, int32_t tile_elems) {
    const int64_t cell_lo = (r.start - r.grid_off) + static_cast<int64_t>(k - r.tile0) * tile_elems;
    const int64_t cell_hi = cell_lo + tile_elems;
    const int64_t end = r.start + r.len;
    const int64_t lo = cell_lo > r.start ? cell_lo : r.start;
    const int64_t hi = cell_hi < end ? cell_hi : end;
    P3TileDesc d;
    d.start = lo;
    d.n = static_cast<int32_t>(hi - lo);
    d.layer = r.layer;
    d.flags = 0;
    d.pad = 0;
    return d;
}

#endif  // P3_TILES_H_
