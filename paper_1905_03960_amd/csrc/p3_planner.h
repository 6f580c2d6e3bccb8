// The slice planner (Sec. 4, Sec. 4.2): integer arithmetic on the host, no GPU
// and no HIP types, so that it is compiled into the library by hipcc and, for
// the host-side checks (address and undefined-behaviour sanitizers), by an
// ordinary C++ compiler.
#ifndef P3_PLANNER_H_
#define P3_PLANNER_H_

#include <stdint.h>

#include <cstring>
#include <vector>

#include "p3.h"
#include "p3_internal.h"

constexpr int64_t kP3AlignElems = 64;      // layer offsets are multiples of 64 elements

struct P3PlanTables {
    int64_t S = 0;
    std::vector<int64_t> n;            // layer sizes
    std::vector<int64_t> offset;       // arena offset of each layer
    std::vector<P3LayerDev> layers;
    std::vector<P3SliceDev> slices;    // start = arena offset
    int64_t N = 0, arena = 0;
    int32_t K = 0, L = 0;              // K: slices this plan owns (all of them unless sharded)
    int32_t n_shards = 1, shard = 0;   // the plan owns the slices whose global id is shard (mod n_shards)
    int32_t K_global = 0;
    std::vector<int32_t> global_id;    // global id of each owned slice (ascending)
};

// Cut every layer into slices of at most slice_elems elements (full ones and one shorter
// remainder), number them by (layer, offset) -- ascending number = descending urgency -- and
// keep those whose number is `shard` modulo n_shards.  Returns a status of p3.h; may throw
// std::bad_alloc.
inline int p3_planner_build(const int64_t* layer_sizes, int32_t n_layers, int64_t slice_elems, int32_t n_shards,
                            int32_t shard, P3PlanTables& t) {
    if (!layer_sizes || n_layers < 1 || slice_elems < 1) return P3_ERR_ARG;
    if (n_shards < 1 || shard < 0 || shard >= n_shards) return P3_ERR_ARG;
    for (int32_t l = 0; l < n_layers; ++l)
        if (layer_sizes[l] < 1) return P3_ERR_ARG;
    // count first so that absurd inputs are refused before anything is allocated
    int64_t K = 0, arena = 0;
    for (int32_t l = 0; l < n_layers; ++l) {
        const int64_t n = layer_sizes[l];
        const int64_t longest = n < slice_elems ? n : slice_elems;
        if (longest > INT32_MAX) return P3_ERR_RANGE;
        K += (n - 1) / slice_elems + 1;
        if (K > INT32_MAX) return P3_ERR_RANGE;
        if (n > INT64_MAX / 8 - arena - kP3AlignElems) return P3_ERR_RANGE;      // arena offsets stay far inside 63 bits
        arena += (n + kP3AlignElems - 1) / kP3AlignElems * kP3AlignElems;
    }
    if (K <= shard) return P3_ERR_RANGE;           // this shard would own nothing
    t.S = slice_elems;
    t.L = n_layers;
    t.K_global = static_cast<int32_t>(K);
    t.n_shards = n_shards;
    t.shard = shard;
    t.n.assign(layer_sizes, layer_sizes + n_layers);
    t.offset.resize(static_cast<size_t>(n_layers));
    t.layers.resize(static_cast<size_t>(n_layers));
    t.slices.clear();
    t.global_id.clear();
    t.slices.reserve(static_cast<size_t>(K / n_shards + 1));
    t.global_id.reserve(static_cast<size_t>(K / n_shards + 1));
    int64_t at = 0, total = 0, g = 0;
    for (int32_t l = 0; l < n_layers; ++l) {
        const int64_t n = layer_sizes[l];
        t.offset[l] = at;
        t.layers[l].first = static_cast<int32_t>(t.slices.size());
        const int64_t k = (n - 1) / slice_elems + 1;
        int64_t own = 0, own_elems = 0;
        // the layer's first slice that this shard owns, then every n_shards-th
        int64_t i = (shard - g % n_shards + n_shards) % n_shards;
        for (; i < k; i += n_shards) {
            P3SliceDev s;
            std::memset(&s, 0, sizeof s);
            s.layer = l;
            // "follows its predecessor in memory": only an unsharded plan owns neighbouring slices
            s.index_in_layer = n_shards == 1 ? static_cast<int32_t>(i) : 0;
            s.start = at + i * slice_elems;
            const int64_t left = n - i * slice_elems;
            s.len = static_cast<int32_t>(left < slice_elems ? left : slice_elems);
            t.slices.push_back(s);
            t.global_id.push_back(static_cast<int32_t>(g + i));
            own += 1;
            own_elems += s.len;
        }
        g += k;
        t.layers[l].count = static_cast<int32_t>(own);
        t.layers[l].elems = own_elems;          // what the layer's completion count has to reach
        for (int64_t j = 0; j < own; ++j) {
            P3SliceDev& s = t.slices[static_cast<size_t>(t.layers[l].first) + static_cast<size_t>(j)];
            s.layer_slices = static_cast<int32_t>(own);
            s.layer_elems = own_elems;
        }
        total += own_elems;
        at += (n + kP3AlignElems - 1) / kP3AlignElems * kP3AlignElems;
    }
    t.K = static_cast<int32_t>(t.slices.size());
    t.N = total;
    t.arena = at;
    return P3_OK;
}

// Upper bound on the tiles of one iteration: tiles are the cells of a grid of `tile`
// elements over the arena clipped to runs of slices; a slice that forms a run of its
// own touches this many cells, and merging neighbours into a run only removes cells.
inline int64_t p3_planner_total_tiles(const P3PlanTables& t, int32_t tile) {
    int64_t n = 0;
    for (const P3SliceDev& s : t.slices) n += p3_run_cells(s.start, s.len, tile);
    return n;
}

// The leading runs of the first selection step of an iteration's first drain in SNAPSHOT mode under the
// priority rule (Sec. 4.2: the most urgent ready slice first; all slices of a marked layer are ready at
// once).  With `marks` the layers marked before the drain, the step claims the `step_slices` lowest-numbered
// ready slices and groups them into runs the way the selector does: a slice continues the run of the slice
// claimed just before it when that slice is its predecessor in the layer's memory.  Writes at most `cap` runs
// (a prefix of the step's runs) and returns how many; 0 for an empty or invalid mark list.
inline int32_t p3_first_step_runs(const P3PlanTables& t, const int32_t* marks, int32_t n_marks, int32_t step_slices,
                                  P3FirstRun* out, int32_t cap) {
    if (!marks || n_marks < 1 || step_slices < 1 || cap < 1) return 0;
    std::vector<char> marked(static_cast<size_t>(t.L), 0);
    for (int32_t i = 0; i < n_marks; ++i) {
        const int32_t l = marks[i];
        if (l < 0 || l >= t.L || marked[static_cast<size_t>(l)]) return 0;
        marked[static_cast<size_t>(l)] = 1;
    }
    int64_t budget = step_slices;
    int32_t n_runs = 0;
    int64_t prev_g = -2, len = 0;
    for (int32_t l = 0; l < t.L && budget > 0; ++l) {
        if (!marked[static_cast<size_t>(l)]) continue;
        const P3LayerDev& ly = t.layers[static_cast<size_t>(l)];
        for (int32_t i = 0; i < ly.count && budget > 0; ++i, --budget) {
            const int64_t g = static_cast<int64_t>(ly.first) + i;
            const P3SliceDev& sl = t.slices[static_cast<size_t>(g)];
            const bool head = !(prev_g + 1 == g && sl.index_in_layer > 0);
            prev_g = g;
            if (head) {
                if (n_runs == cap) return n_runs;          // a prefix of the step is enough
                out[n_runs].start = sl.start;
                out[n_runs].layer = sl.layer;
                len = 0;
                n_runs += 1;
            }
            len += sl.len;
            // the workers turn these records into addresses without looking at them again: nothing leaves here
            // that is not inside the arena (and a run longer than the length field is left out)
            if (sl.start < 0 || sl.len < 1 || sl.start > t.arena || sl.len > t.arena - sl.start ||
                len > static_cast<int64_t>(UINT32_MAX))
                return n_runs - 1;
            out[n_runs - 1].len = static_cast<uint32_t>(len);
        }
    }
    return n_runs;
}

#endif  // P3_PLANNER_H_
