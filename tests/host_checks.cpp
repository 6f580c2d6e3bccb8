// Host-side check driver, built by tests/test_host_sanitized.py with
// g++ -fsanitize=address,undefined: runs the library's host-only integer logic
// (slice planner, run/tile arithmetic -- the same headers the gfx950 build
// compiles) and the CPU oracle (oracle/p3_oracle.cpp, linked in) on inputs read
// from stdin, on exactly-sized heap buffers, and prints what they return.  The
// Python test compares the output with pins and with brute force; a sanitizer
// report fails the run.  TEST INFRASTRUCTURE ONLY.
//
// One command per line:
//   plan  n_shards shard S L n_0..n_{L-1}
//   tiles start len layer tile0 tile_elems
//   valid start len grid_off layer tile0 tile_end arena_elems n_layers tile_elems
//   oplan S L n_0..n_{L-1}
//   osnap n e_0..        | oticked r_0..r_{L-1} | ofifo r_0..r_{L-1}
//   oreplay n_marks m.. n_claims s..
//   oapply W dtype lr mu rescale wd n_order o.. then W*N gradient words, N weight words, N momentum words (hex)
#include <cinttypes>
#include <cstdio>
#include <cstdlib>
#include <iostream>
#include <sstream>
#include <string>
#include <vector>

#include "p3_planner.h"

extern "C" {
void* p3o_plan_create(const int64_t* layer_sizes, int32_t n_layers, int64_t S);
void p3o_plan_destroy(void* h);
int32_t p3o_num_slices(const void* h);
int32_t p3o_num_layers(const void* h);
int64_t p3o_num_elems(const void* h);
int32_t p3o_slice_info(const void* h, int32_t g, int32_t* layer, int64_t* offset, int64_t* len);
int32_t p3o_order_snapshot(const void* h, const int32_t* events, int32_t n_events, int32_t* out, int32_t cap);
int32_t p3o_order_ticked(const void* h, const int64_t* release, int32_t* out, int64_t* claim_tick, int32_t cap);
int32_t p3o_order_ticked_fifo(const void* h, const int64_t* release, int32_t* out, int64_t* claim_tick, int32_t cap);
int32_t p3o_order_replay(const void* h, const int32_t* marks, int32_t n_marks, const int32_t* seen, int32_t n_claims,
                         int32_t* out);
int32_t p3o_apply(const void* h, const int32_t* order, int32_t n_order, int32_t W, const void* const* grads,
                  int32_t dtype, float* w, float* m, float lr, float mu, float rescale, float wd);
}

namespace {

template <class T>
std::vector<T> read_n(std::istringstream& in, size_t n) {
    std::vector<T> v(n);
    for (size_t i = 0; i < n; ++i) {
        long long x = 0;
        in >> x;
        v[i] = static_cast<T>(x);
    }
    return v;
}

template <class T>
void print_vec(const char* tag, const T* v, int32_t n) {
    std::printf("%s %d", tag, n);
    for (int32_t i = 0; i < n; ++i) std::printf(" %lld", static_cast<long long>(v[i]));
    std::printf("\n");
}

}  // namespace

int main() {
    void* oplan = nullptr;
    std::string line;
    while (std::getline(std::cin, line)) {
        std::istringstream in(line);
        std::string cmd;
        if (!(in >> cmd)) continue;
        if (cmd == "plan") {
            long long n_shards, shard, S, L;
            in >> n_shards >> shard >> S >> L;
            std::vector<int64_t> sizes = read_n<int64_t>(in, L > 0 ? static_cast<size_t>(L) : 0);
            P3PlanTables t;
            const int rc = p3_planner_build(sizes.data(), static_cast<int32_t>(L), S, static_cast<int32_t>(n_shards),
                                            static_cast<int32_t>(shard), t);
            std::printf("plan %d %d %lld %lld %d\n", rc, t.K, static_cast<long long>(t.N),
                        static_cast<long long>(t.arena), t.K_global);
            if (rc != P3_OK) continue;
            for (int32_t g = 0; g < t.K; ++g) {
                const P3SliceDev& s = t.slices[static_cast<size_t>(g)];
                std::printf("s %d %lld %d %d %d %d %lld\n", s.layer, static_cast<long long>(s.start), s.len,
                            t.global_id[static_cast<size_t>(g)], s.layer_slices, s.index_in_layer,
                            static_cast<long long>(s.layer_elems));
            }
            for (int32_t l = 0; l < t.L; ++l)
                std::printf("l %d %d %lld %lld\n", t.layers[l].first, t.layers[l].count,
                            static_cast<long long>(t.layers[l].elems), static_cast<long long>(t.offset[l]));
            std::printf("tiles3328 %lld\n", static_cast<long long>(p3_planner_total_tiles(t, 3328)));
        } else if (cmd == "first") {
            // first <n_shards> <shard> <S> <step_slices> <cap> <L> sizes... <n_marks> marks...
            long long n_shards, shard, S, step, cap, L, n_marks;
            in >> n_shards >> shard >> S >> step >> cap >> L;
            std::vector<int64_t> sizes = read_n<int64_t>(in, L > 0 ? static_cast<size_t>(L) : 0);
            in >> n_marks;
            std::vector<int32_t> marks = read_n<int32_t>(in, n_marks > 0 ? static_cast<size_t>(n_marks) : 0);
            P3PlanTables t;
            const int rc = p3_planner_build(sizes.data(), static_cast<int32_t>(L), S, static_cast<int32_t>(n_shards),
                                            static_cast<int32_t>(shard), t);
            if (rc != P3_OK) {
                std::printf("first %d 0\n", rc);
                continue;
            }
            std::vector<P3FirstRun> runs(static_cast<size_t>(cap > 0 ? cap : 1));   // exactly cap: an overrun is reported
            const int32_t n = p3_first_step_runs(t, marks.data(), static_cast<int32_t>(n_marks), static_cast<int32_t>(step),
                                                 runs.data(), static_cast<int32_t>(cap));
            std::printf("first 0 %d\n", n);
            for (int32_t r = 0; r < n; ++r)
                std::printf("r %lld %u %d\n", static_cast<long long>(runs[static_cast<size_t>(r)].start),
                            runs[static_cast<size_t>(r)].len, runs[static_cast<size_t>(r)].layer);
        } else if (cmd == "tiles") {
            long long start, len, layer, tile0, tile;
            in >> start >> len >> layer >> tile0 >> tile;
            P3Run r;
            r.start = start;
            r.len = len;
            r.grid_off = static_cast<int32_t>(start % tile);
            r.layer = static_cast<int32_t>(layer);
            r.tile0 = static_cast<uint32_t>(tile0);
            const int64_t cells = p3_run_cells(start, len, static_cast<int32_t>(tile));
            r.tile_end = static_cast<uint32_t>(tile0 + cells);
            std::printf("cells %lld\n", static_cast<long long>(cells));
            for (uint32_t k = r.tile0; k != r.tile_end; ++k) {
                const P3TileDesc d = p3_tile_of_run(r, k, static_cast<int32_t>(tile));
                std::printf("t %lld %d %d\n", static_cast<long long>(d.start), d.n, d.layer);
            }
        } else if (cmd == "valid") {
            long long start, len, grid_off, layer, tile0, tile_end, arena, nl, tile;
            in >> start >> len >> grid_off >> layer >> tile0 >> tile_end >> arena >> nl >> tile;
            P3Run r;
            r.start = start;
            r.len = len;
            r.grid_off = static_cast<int32_t>(grid_off);
            r.layer = static_cast<int32_t>(layer);
            r.tile0 = static_cast<uint32_t>(tile0);
            r.tile_end = static_cast<uint32_t>(tile_end);
            std::printf("valid %d\n", p3_run_valid(r, arena, static_cast<int32_t>(nl), static_cast<int32_t>(tile)) ? 1 : 0);
        } else if (cmd == "oplan") {
            long long S, L;
            in >> S >> L;
            std::vector<int64_t> sizes = read_n<int64_t>(in, static_cast<size_t>(L));
            if (oplan) p3o_plan_destroy(oplan);
            oplan = p3o_plan_create(sizes.data(), static_cast<int32_t>(L), S);
            if (!oplan) {
                std::printf("oplan -1\n");
                continue;
            }
            const int32_t K = p3o_num_slices(oplan);
            std::printf("oplan %d %lld\n", K, static_cast<long long>(p3o_num_elems(oplan)));
            for (int32_t g = 0; g < K; ++g) {
                int32_t layer = 0;
                int64_t off = 0, len = 0;
                p3o_slice_info(oplan, g, &layer, &off, &len);
                std::printf("o %d %lld %lld\n", layer, static_cast<long long>(off), static_cast<long long>(len));
            }
        } else if (cmd == "osnap" && oplan) {
            long long n;
            in >> n;
            std::vector<int32_t> ev = read_n<int32_t>(in, static_cast<size_t>(n));
            const int32_t K = p3o_num_slices(oplan);
            std::vector<int32_t> out(static_cast<size_t>(K));
            const int32_t got = p3o_order_snapshot(oplan, ev.data(), static_cast<int32_t>(n), out.data(), K);
            print_vec("order", out.data(), got < 0 ? 0 : got);
        } else if ((cmd == "oticked" || cmd == "ofifo") && oplan) {
            const int32_t K = p3o_num_slices(oplan), L = p3o_num_layers(oplan);
            std::vector<int64_t> rel = read_n<int64_t>(in, static_cast<size_t>(L));
            std::vector<int32_t> out(static_cast<size_t>(K));
            std::vector<int64_t> tick(static_cast<size_t>(K));
            const int32_t got = cmd == "oticked" ? p3o_order_ticked(oplan, rel.data(), out.data(), tick.data(), K)
                                                 : p3o_order_ticked_fifo(oplan, rel.data(), out.data(), tick.data(), K);
            print_vec("order", out.data(), got < 0 ? 0 : got);
            print_vec("ticks", tick.data(), got < 0 ? 0 : got);
        } else if (cmd == "oreplay" && oplan) {
            long long nm, nc;
            in >> nm;
            std::vector<int32_t> marks = read_n<int32_t>(in, static_cast<size_t>(nm));
            in >> nc;
            std::vector<int32_t> seen = read_n<int32_t>(in, static_cast<size_t>(nc));
            std::vector<int32_t> out(static_cast<size_t>(nc));
            const int32_t got = p3o_order_replay(oplan, marks.data(), static_cast<int32_t>(nm), seen.data(),
                                                 static_cast<int32_t>(nc), out.data());
            std::printf("replay %d\n", got);
            print_vec("order", out.data(), got < 0 ? 0 : got);
        } else if (cmd == "oapply" && oplan) {
            long long W, dtype, n_order;
            double lr, mu, rescale, wd;
            in >> W >> dtype >> lr >> mu >> rescale >> wd >> n_order;
            std::vector<int32_t> order = read_n<int32_t>(in, static_cast<size_t>(n_order));
            const int64_t N = p3o_num_elems(oplan);
            auto hex_word = [&in]() {
                std::string h;
                in >> h;
                return static_cast<uint32_t>(std::strtoul(h.c_str(), nullptr, 16));
            };
            // exactly-sized buffers: N elements of 4 (fp32) or 2 (bf16) bytes per copy
            std::vector<std::vector<uint8_t>> g(static_cast<size_t>(W));
            std::vector<const void*> gp(static_cast<size_t>(W));
            for (long long k = 0; k < W; ++k) {
                g[k].resize(static_cast<size_t>(N) * (dtype == 0 ? 4 : 2));
                for (int64_t e = 0; e < N; ++e) {
                    const uint32_t v = hex_word();
                    if (dtype == 0) reinterpret_cast<uint32_t*>(g[k].data())[e] = v;
                    else reinterpret_cast<uint16_t*>(g[k].data())[e] = static_cast<uint16_t>(v);
                }
                gp[k] = g[k].data();
            }
            std::vector<float> w(static_cast<size_t>(N)), m(static_cast<size_t>(N));
            for (int64_t e = 0; e < N; ++e) reinterpret_cast<uint32_t*>(w.data())[e] = hex_word();
            for (int64_t e = 0; e < N; ++e) reinterpret_cast<uint32_t*>(m.data())[e] = hex_word();
            const int32_t rc = p3o_apply(oplan, order.data(), static_cast<int32_t>(n_order), static_cast<int32_t>(W),
                                         gp.data(), static_cast<int32_t>(dtype), w.data(), m.data(),
                                         static_cast<float>(lr), static_cast<float>(mu), static_cast<float>(rescale),
                                         static_cast<float>(wd));
            std::printf("apply %d\n", rc);
            std::printf("w");
            for (int64_t e = 0; e < N; ++e) std::printf(" %08x", reinterpret_cast<uint32_t*>(w.data())[e]);
            std::printf("\nm");
            for (int64_t e = 0; e < N; ++e) std::printf(" %08x", reinterpret_cast<uint32_t*>(m.data())[e]);
            std::printf("\n");
        } else {
            std::printf("error unknown-or-out-of-order %s\n", cmd.c_str());
        }
    }
    if (oplan) p3o_plan_destroy(oplan);
    std::printf("end\n");
    return 0;
}
