// Host-only exercise of the library's CPU-side logic, built with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host code (tests/test_sanitizers.py builds and runs it; no
// GPU is touched: every launch is either rejected by argument checks or refused by the library's
// own launch-failure seam before it reaches the runtime).
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <map>
#include <utility>
#include <vector>

#include "amulet.h"
#include "amulet_internal.h"

#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            exit(1);                                                       \
        }                                                                  \
    } while (0)

struct Grid {
    int n0, n1;
    std::vector<double> t;
    int calls;
};
static double grid_score(int i0, int i1, void *ctx)
{
    Grid *g = (Grid *)ctx;
    CHECK(i0 >= 0 && i0 < g->n0 && i1 >= 0 && i1 < g->n1);
    g->calls++;
    return g->t[(size_t)i0 * g->n1 + i1];
}

int main()
{
    // ---- the two-stage greedy search on grids of every small size, with pseudo-random scores
    uint32_t seed = 12345u;
    for (int n0 = 1; n0 <= 7; ++n0)
        for (int n1 = 1; n1 <= 7; ++n1) {
            Grid g{n0, n1, std::vector<double>((size_t)n0 * n1), 0};
            for (double &x : g.t) { seed = seed * 1664525u + 1013904223u; x = (double)(seed >> 8); }
            int b0 = -1, b1 = -1;
            const int calls = amulet_greedy_search(n0, n1, grid_score, &g, &b0, &b1);
            CHECK(calls == g.calls && calls >= n0 && calls <= n0 + n1 - 1);
            CHECK(b0 >= 0 && b0 < n0 && b1 >= 0 && b1 < n1);
            for (int i = 0; i < n0; ++i) CHECK(g.t[(size_t)b0 * n1] <= g.t[(size_t)i * n1]);   // stage 1 keeps the minimum
            for (int j = 1; j <= b1; ++j) CHECK(g.t[(size_t)b0 * n1 + j] <= g.t[(size_t)b0 * n1 + j - 1]);   // stage 2 never climbs
        }
    int b0, b1;
    CHECK(amulet_greedy_search(0, 3, grid_score, nullptr, &b0, &b1) == AMULET_ERR_DIM);
    CHECK(amulet_greedy_search(2, 2, nullptr, nullptr, &b0, &b1) == AMULET_ERR_NULL);

    // ---- the register rule over a range of kernels
    for (int h = 1; h <= 16; ++h)
        for (int w = 1; w <= 64; w += 5)
            for (int sw = 1; sw <= 16; sw *= 2) {
                const int need = amulet_register_demand(h, w, sw, 1, 1, 2, 1, 3);
                CHECK(need > h * ((w + sw - 1) / sw));
                const int hh = amulet_choose_kernel_height(h, w, sw, 1, 1, 2, 1, 3, need);
                CHECK(hh == h);
            }
    CHECK(amulet_register_demand(0, 1, 1, 0, 0, 0, 0, 0) == AMULET_ERR_DIM);

    // ---- the XCD-aware tile order: every tile exactly once, padding owns nothing
    for (int64_t tm = 1; tm <= 70; tm += 3)
        for (int64_t tn = 1; tn <= 40; tn += 7) {
            const int64_t grid = amulet_tile_grid(tm, tn);
            CHECK(grid % 8 == 0 && grid >= tm * tn);
            std::map<std::pair<int64_t, int64_t>, int> seen;
            for (int64_t b = 0; b < grid; ++b) {
                int64_t m = -1, n = -1;
                const int rc = amulet_tile_of_workgroup(b, tm, tn, &m, &n);
                CHECK(rc == 0 || rc == 1);
                if (rc == 1) { CHECK(m >= 0 && m < tm && n >= 0 && n < tn); seen[{m, n}]++; }
            }
            CHECK((int64_t)seen.size() == tm * tn);
            for (auto &kv : seen) CHECK(kv.second == 1);
        }
    int64_t m, n;
    CHECK(amulet_tile_of_workgroup(1LL << 40, 4, 4, &m, &n) == AMULET_ERR_DIM);
    CHECK(amulet_tile_of_workgroup(0, 4, 4, nullptr, &n) == AMULET_ERR_NULL);

    // ---- launch plans: tail split and full split over many sizes (pure host arithmetic)
    for (int64_t real = 1; real <= 5000; real += 37)
        for (int64_t round : {256LL, 512LL, 1024LL})
            for (int64_t K : {64LL, 500LL, 512LL, 1000LL, 4096LL, 100000LL, 2147418111LL}) {
                amulet::TailSplit t;
                const int64_t wgs = amulet::xcd_grid(real, 1);
                if (amulet::choose_tail_split(real, wgs, round, K, 64, t)) {
                    CHECK(t.splits >= 2 && t.splits <= 8 && t.chunk % 64 == 0);
                    CHECK((int64_t)t.chunk * t.splits >= K && (int64_t)t.chunk * (t.splits - 1) < K);
                    CHECK(t.base >= 0 && t.base < real && t.blocks == wgs - t.base && t.grid == t.base + t.blocks * t.splits);
                }
                static const double rate[3] = {0.72, 0.81, 1.0};
                const int sp = amulet::choose_full_split(real, 32, K, rate, 3);
                CHECK(sp >= 1 && sp <= 8 && (sp == 1 || K / sp >= 256 / 2));
            }

    // ---- packing helpers
    for (int eb : {1, 4, 8})
        for (int64_t cols : {1LL, 31LL, 4096LL, 65536LL, 1LL << 30}) {
            const int64_t ld = amulet_packed_ld(cols, eb);
            CHECK(ld >= cols && !amulet_pitch_collides(ld, eb));
        }
    CHECK(amulet_count_i8_repack_workspace_bytes(100, 200, 300) > 0 && amulet_count_i8_workspace_bytes(1, 1, 0, 5, 5) == 0);

    // ---- argument checks of the compute calls (the pointers are never dereferenced on the host)
    float *fp = (float *)(uintptr_t)4096;
    int8_t *bp = (int8_t *)(uintptr_t)4096;
    int32_t *ip = (int32_t *)(uintptr_t)4096;
    CHECK(amulet_mmlike_f32(9, 1, 1, 1, fp, 1, fp, 1, fp, fp, 1, nullptr) == AMULET_ERR_TASK);
    CHECK(amulet_mmlike_f32(1, -1, 1, 1, fp, 1, fp, 1, fp, fp, 1, nullptr) == AMULET_ERR_DIM);
    CHECK(amulet_mmlike_f32(1, 2, 3, 4, fp, 3, fp, 3, fp, fp, 3, nullptr) == AMULET_ERR_LD);
    CHECK(amulet_mmlike_f32(1, 1LL << 31, 3, 4, fp, 4, fp, 3, fp, fp, 3, nullptr) == AMULET_ERR_RANGE);
    CHECK(amulet_mmlike_f32(1, 0, 3, 4, nullptr, 4, nullptr, 3, nullptr, nullptr, 3, nullptr) == AMULET_OK);
    CHECK(amulet_count_i8(2, 3, 4, bp, 3, bp, 3, ip, 3, nullptr) == AMULET_ERR_LD);
    CHECK(amulet_count_i8_static(0, 0, 8191, 8191, 4095, bp, 4095, bp, 8191, ip, 8191, nullptr) == AMULET_ERR_WORKSPACE);
    CHECK(amulet_tune(55, 8, 8, 8, nullptr) == AMULET_ERR_TASK);
    CHECK(amulet_count_i8_adaptive(2, 3, 4, bp, 3, bp, 3, ip, 3, nullptr, nullptr, nullptr) == AMULET_ERR_LD);
    amulet_debug_fail_launches(1);
    CHECK(amulet_count_i8_adaptive(12288, 16384, 128, bp, 128, bp, 16384, ip, 16384, nullptr, nullptr, nullptr) == AMULET_ERR_LAUNCH);

    // ---- every vector-ALU launch plan, refused at the launch: shapes x tasks x forms x layouts x sizes
    const int64_t sizes[][3] = {{1, 1, 1}, {300, 700, 200}, {8192, 8192, 8192}, {770, 6100, 1100}, {64, 64, 100000},
                                {2147418111LL, 64, 4}, {64, 2147418111LL, 4}, {4096, 4096, 65536}};
    for (auto &sz : sizes)
        for (int task = 1; task <= 3; ++task)
            for (int shape = -1; shape < amulet_shape_count(task); ++shape)
                for (int form = 0; form < 4; ++form)
                    for (int layout = 0; layout < 4; ++layout) {
                        const int ta = layout & 1, tb = layout >> 1;
                        const int64_t M = sz[0], N = sz[1], K = sz[2];
                        amulet_debug_fail_launches(1);
                        const int rc = amulet_mmlike_f32_general(task, form, ta, tb, shape, M, N, K, fp, ta ? M : K, fp,
                                                                 tb ? K : N, fp, N, fp, fp, N, nullptr);
                        CHECK(rc == AMULET_ERR_LAUNCH);
                    }
    // ---- the streamed identity kernels' K-split model over many sizes
    for (int64_t part = 1; part <= 700; part += 3)
        for (int64_t K : {16LL, 128LL, 500LL, 1024LL, 4096LL, 100000LL, 2147418111LL})
            for (int cap : {2, 3}) {
                static const double rate3[3] = {0.92, 0.985, 1.0}, rate2[2] = {0.93, 1.0};
                const int sp = amulet::choose_stream_split(part, 32, K, cap, cap == 3 ? rate3 : rate2);
                CHECK(sp >= 1 && sp <= 1024 && (sp == 1 || K / sp >= 128));
            }
    // ---- a k range of the streamed identity kernels never ends in less than a stage
    for (int64_t K = 16; K <= 3000; ++K)
        for (int sp = 2; sp <= 40; ++sp) {
            const int64_t c0 = ((K + sp - 1) / sp + 15) / 16 * 16;
            const int64_t chunk = amulet::chunk_with_a_whole_last_stage(K, c0, 16);
            CHECK(chunk >= c0 && chunk % 16 == 0);
            CHECK(chunk >= K || K % chunk == 0 || K % chunk >= 16);
        }
    CHECK(amulet::chunk_with_a_whole_last_stage(1028, 128, 16) == 144);   // 1028 = 8 x 128 + 4
    // ---- every identity launch plan (vector-ALU shapes, both matrix-core tiles, the streamed
    // kernel and what it falls back to), fp32 and fp64, refused at the launch
    const int64_t id_sizes[][3] = {{1, 1, 1}, {300, 700, 200}, {4096, 4096, 4096}, {2048, 2048, 2048}, {1408, 3200, 1104},
                                   {128, 256, 100000}, {1536, 1536, 4096}, {8192, 8192, 8192}, {2147418111LL, 128, 16},
                                   {4000, 4100, 4004}, {128, 256, 1028}, {1300, 3204, 1108}};
    double *dp = (double *)(uintptr_t)4096;
    for (auto &sz : id_sizes)
        for (int layout = 0; layout < 4; ++layout) {
            const int ta = layout & 1, tb = layout >> 1;
            const int64_t M = sz[0], N = sz[1], K = sz[2];
            for (int shape = -1; shape < amulet_shape_count(0); ++shape) {
                amulet_debug_fail_launches(1);
                CHECK(amulet_mmlike_f32_general(0, 0, ta, tb, shape, M, N, K, fp, ta ? M : K, fp, tb ? K : N, nullptr, 0,
                                                nullptr, fp, N, nullptr) == AMULET_ERR_LAUNCH);
            }
            for (int task = 0; task <= 3; ++task)
                for (int shape = -1; shape < amulet_f64_shape_count(); ++shape) {
                    amulet_debug_fail_launches(1);
                    CHECK(amulet_mmlike_f64_shape(task, shape, (task + shape + 4) % 4, ta, tb, M, N, K, dp, ta ? M : K, dp,
                                                  tb ? K : N, dp, N, dp, dp, N, nullptr) == AMULET_ERR_LAUNCH);
                }
        }
    CHECK(amulet_mmlike_f64_shape(1, 6, 0, 0, 0, 8, 8, 8, dp, 8, dp, 8, dp, 8, dp, dp, 8, nullptr) == AMULET_ERR_SHAPE);
    CHECK(amulet_selected_shape_f64(9, 8, 8, 8) == AMULET_ERR_TASK);
    amulet_debug_fail_launches(0);
    CHECK(amulet_get_deterministic() == 0 || amulet_get_deterministic() == 1);
    amulet_set_deterministic(1);
    CHECK(amulet_get_deterministic() == 1);
    amulet_set_deterministic(0);
    printf("host logic under sanitizers: ok\n");
    return 0;
}
