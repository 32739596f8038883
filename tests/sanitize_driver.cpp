// Host code under AddressSanitizer / UndefinedBehaviorSanitizer (CPU only): the host half of libepara
// (planner, scheduler, handler, placement, simulator) and the C oracle, driven over seeded inputs that
// include the edge cases (nothing to do, empty groups, arrays that are too small).  Built and run by
// tests/test_sanitizers.py; any sanitizer report makes the process exit non-zero.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "epara.h"

extern "C" {
void oracle_dense_forward(const double* X, const double* W, const double* b, int64_t M, int64_t K, int64_t N, double s, int act, double* Y);
void oracle_swiglu_hidden(const double* X, const double* Wg, const double* Wu, int64_t M, int64_t K, int64_t F, double sg, double su, double* H);
void oracle_bf16_decode(const uint16_t* src, int64_t n, double* dst);
void oracle_bf16_encode(const float* src, int64_t n, uint16_t* dst);
void oracle_e4m3_decode(const uint8_t* src, int64_t n, double scale, double* dst);
void oracle_e4m3_encode(const double* src, int64_t n, double scale, uint8_t* dst);
void oracle_act_array(const double* z, int64_t n, int act, double* out);
}

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t next_u64() { rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17; return rng_state; }
static int32_t rnd(int32_t lo, int32_t hi) { return lo + static_cast<int32_t>(next_u64() % static_cast<uint64_t>(hi - lo + 1)); }
static double unit() { return static_cast<double>(next_u64() >> 11) / 9007199254740992.0; }

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); return 1; } } while (0)

static double coverage_phi(const int32_t* p, int32_t n, void* user)
{
    const int32_t* weights = static_cast<const int32_t*>(user);
    bool seen[16] = {};
    double v = 0;
    for (int32_t i = 0; i < n; ++i) if (!seen[p[i] % 16]) { seen[p[i] % 16] = true; v += weights[p[i] % 16]; }
    return v;
}

int main()
{
    // ---- planner, scheduler, chain waits over random launches (both class tables, gated and plain)
    for (int round = 0; round < 60; ++round) {
        const int32_t G = rnd(0, 9), dtype = round % 3 == 0 ? EPARA_F32 : (round % 3 == 1 ? EPARA_BF16 : EPARA_FP8_E4M3);
        const int32_t gated = dtype != EPARA_F32 && round % 2;
        std::vector<epara_group_desc> groups(static_cast<size_t>(G));
        for (auto& g : groups) { g.M = rnd(0, 3) == 0 ? 0 : rnd(1, 700); g.K = 8 * rnd(1, 40); g.N = rnd(1, 600); g.act = gated ? EPARA_ACT_SWIGLU : rnd(0, 4); g.has_bias = rnd(0, 1); g.category = rnd(0, 1); }
        epara_tile_class classes[4];
        int32_t nc = 0, ns = 0;
        CHECK(epara_kernel_classes(dtype, gated, round % 5 == 0 && dtype != EPARA_F32, classes, 4, &nc, &ns) == EPARA_OK);
        int64_t n_tiles = -1;
        std::vector<int64_t> row_off(G + 1), x_off(G + 1), y_off(G + 1);
        CHECK(epara_plan_groups(groups.data(), G, classes, nc, row_off.data(), x_off.data(), y_off.data(), nullptr, 0, &n_tiles) == EPARA_OK);
        std::vector<epara_tile> tiles(static_cast<size_t>(n_tiles));
        if (n_tiles > 0) {
            int64_t again = 0;
            CHECK(epara_plan_groups(groups.data(), G, classes, nc, nullptr, nullptr, nullptr, tiles.data(), n_tiles - 1, &again) == EPARA_ERR_CAPACITY);
        }
        CHECK(epara_plan_groups(groups.data(), G, classes, nc, nullptr, nullptr, nullptr, tiles.data(), n_tiles, &n_tiles) == EPARA_OK);
        const int32_t W = 8 * rnd(1, 32), X = 8;
        int64_t n_slots = 0;
        CHECK(epara_schedule_tiles(groups.data(), G, classes, nc, ns, tiles.data(), n_tiles, W, X, 1, 4, nullptr, 0, &n_slots) == EPARA_OK);
        std::vector<int32_t> order(static_cast<size_t>(n_slots));
        CHECK(epara_schedule_tiles(groups.data(), G, classes, nc, ns, tiles.data(), n_tiles, W, X, rnd(1, 3), rnd(1, 5), order.data(), n_slots, &n_slots) == EPARA_OK);
        std::vector<char> seen(static_cast<size_t>(n_tiles), 0);
        for (int32_t t : order) if (t >= 0) { CHECK(t < n_tiles && !seen[t]); seen[t] = 1; }
        for (char c : seen) CHECK(c);
        epara_phase_schedule ph[2] = {};
        std::vector<int32_t> o2[2];
        for (int p = 0; p < 2; ++p) { ph[p].groups = groups.data(); ph[p].classes = classes; ph[p].tiles = tiles.data(); ph[p].n_tiles = n_tiles; ph[p].G = G; ph[p].n_classes = nc; ph[p].n_stream_classes = ns; }
        CHECK(epara_schedule_chain(ph, 2, W, X, 1, 4) == EPARA_OK);
        for (int p = 0; p < 2; ++p) { o2[p].resize(static_cast<size_t>(ph[p].n_slots)); ph[p].order = o2[p].data(); ph[p].order_cap = ph[p].n_slots; }
        CHECK(epara_schedule_chain(ph, 2, W, X, 1, 4) == EPARA_OK);
        std::vector<int32_t> producer(static_cast<size_t>(G));
        for (auto& q : producer) q = G ? rnd(-1, G - 1) : -1;
        std::vector<epara_chain_wait> waits(static_cast<size_t>(G));
        CHECK(epara_chain_waits(tiles.data(), n_tiles, G, 3, producer.data(), G, waits.data()) == EPARA_OK);
    }
    // ---- the whole planning decision from C alone: the decode and prefill FFN launches, singly and as chains;
    // every tile of the chosen plan exactly once in the order, every group covered by its tiles
    {
        const int32_t rows4[4] = {1, 8, 32, 64}, rows5[2] = {4692, 3500};
        for (int mix = 4; mix <= 5; ++mix) {
            const int32_t G = mix == 4 ? 4 : 2, d = mix == 4 ? 4096 : 5120, f = mix == 4 ? 11008 : 13824;
            std::vector<epara_group_desc> up(G), down(G);
            for (int32_t g = 0; g < G; ++g) {
                const int32_t M = mix == 4 ? rows4[g] : rows5[g];
                up[g] = {M, d, f, EPARA_ACT_SWIGLU, 0, 0};
                down[g] = {M, f, d, EPARA_ACT_NONE, 0, 0};
            }
            for (int which = 0; which < 2; ++which) {
                const std::vector<epara_group_desc>& groups = which ? down : up;
                epara_launch_plan plan;
                CHECK(epara_plan_launch(groups.data(), G, EPARA_BF16, 256, 8, 1, 4, nullptr, nullptr, nullptr, nullptr, 0, nullptr, 0, nullptr, &plan) == EPARA_OK);
                std::vector<epara_tile> tiles(static_cast<size_t>(plan.n_tiles));
                std::vector<int32_t> order(static_cast<size_t>(plan.n_slots));
                std::vector<int64_t> row_off(G + 1);
                std::vector<int32_t> split_base(static_cast<size_t>(G));
                CHECK(epara_plan_launch(groups.data(), G, EPARA_BF16, 256, 8, 1, 4, row_off.data(), nullptr, nullptr, tiles.data(), plan.n_tiles - 1,
                                        order.data(), plan.n_slots, split_base.data(), &plan) == EPARA_ERR_CAPACITY);
                CHECK(epara_plan_launch(groups.data(), G, EPARA_BF16, 256, 8, 1, 4, row_off.data(), nullptr, nullptr, tiles.data(), plan.n_tiles,
                                        order.data(), plan.n_slots, split_base.data(), &plan) == EPARA_OK);
                CHECK(plan.gated == (which ? 0 : 1) && plan.n_classes == 4 && plan.makespan > 0);
                std::vector<int64_t> area(static_cast<size_t>(G), 0);
                for (const epara_tile& t : tiles) { CHECK(t.rows >= 1 && t.cols >= 1 && t.m0 + t.rows <= groups[t.group].M && t.n0 + t.cols <= groups[t.group].N); area[t.group] += static_cast<int64_t>(t.rows) * t.cols; }
                for (int32_t g = 0; g < G; ++g) CHECK(area[g] == static_cast<int64_t>(groups[g].M) * groups[g].N);
                std::vector<int32_t> seen(tiles.size(), 0), parts(tiles.size(), 0);   // bit j of seen[t]: part j of tile t was visited
                for (int32_t e : order) if (e >= 0) {
                    const int32_t t = EPARA_ORDER_TILE(e), j = (e >> 24) & 15, n = (e >> 28) + 1;
                    CHECK(static_cast<size_t>(t) < tiles.size() && j < n && !(seen[t] >> j & 1) && (parts[t] == 0 || parts[t] == n));
                    seen[t] |= 1 << j; parts[t] = n;
                }
                int32_t n_split = 0, n_panel = 0, panel_parts = 1, panel_more = 0;
                CHECK(epara_panel_split(groups.data(), G, plan.classes, plan.n_classes, plan.n_stream_classes, 256, &n_panel, &panel_parts, &panel_more) == EPARA_OK);
                for (size_t t = 0; t < tiles.size(); ++t) {
                    const epara_tile_class& c = plan.classes[tiles[t].cls];
                    int32_t want = tiles[t].cls < plan.n_stream_classes && c.split_K > 0 && groups[tiles[t].group].K >= c.split_K ? EPARA_SPLIT_PARTS : 1;
                    if (tiles[t].cls >= plan.n_stream_classes && static_cast<int64_t>(t) >= plan.n_tiles - plan.n_panel_split_tiles)
                        want = panel_parts + (static_cast<int64_t>(t) >= plan.n_tiles - panel_more ? 1 : 0);
                    CHECK(parts[t] == want && seen[t] == (1 << want) - 1);
                    n_split += want > 1 && tiles[t].cls < plan.n_stream_classes;
                }
                CHECK(plan.n_split_tiles == n_split && plan.n_panel_split_tiles == n_panel);
                CHECK(plan.workspace_bytes == epara_split_workspace_bytes(n_split, n_panel));
                CHECK(epara_workspace_bytes(groups.data(), G, EPARA_BF16, 256) >= plan.workspace_bytes);
                if (mix == 5 && which == 1) CHECK(n_panel == 148 && panel_parts == 3 && panel_more == 68);
            }
            const int32_t producer[4] = {0, 1, 2, 3};
            epara_chain_plan_phase ph[2];
            std::memset(ph, 0, sizeof ph);
            ph[0].groups = up.data(); ph[0].G = G; ph[1].groups = down.data(); ph[1].G = G; ph[1].producer = producer;
            int64_t finish = 0;
            CHECK(epara_plan_chain(ph, 2, EPARA_BF16, 256, 8, 1, 4, &finish) == EPARA_OK && finish > 0);
            std::vector<epara_tile> ct[2];
            std::vector<int32_t> co[2];
            std::vector<epara_chain_wait> waits(static_cast<size_t>(G));
            for (int p = 0; p < 2; ++p) {
                ct[p].resize(static_cast<size_t>(ph[p].plan.n_tiles)); co[p].resize(static_cast<size_t>(ph[p].plan.n_slots));
                ph[p].tiles = ct[p].data(); ph[p].tiles_cap = ph[p].plan.n_tiles; ph[p].order = co[p].data(); ph[p].order_cap = ph[p].plan.n_slots;
            }
            ph[1].waits = waits.data();
            CHECK(epara_plan_chain(ph, 2, EPARA_BF16, 256, 8, 1, 4, &finish) == EPARA_OK);
            CHECK(ph[0].counter_base == 0 && ph[1].counter_base == G);
            for (int32_t g = 0; g < G; ++g) {
                int32_t n = 0;
                for (const epara_tile& t : ct[0]) n += t.group == g;
                CHECK(waits[g].counter == g && waits[g].need == n);
            }
        }
    }
    // ---- batch accounting, segments, dealer
    {
        const int32_t rows[7] = {3, 0, 5, 1, 9, 2, 2};
        const int64_t off[4] = {0, 2, 2, 7};
        int32_t M[3];
        int64_t first[7];
        CHECK(epara_batch_rows(rows, off, 3, M, first) == EPARA_OK && M[0] == 3 && M[1] == 0 && M[2] == 19);
        const int64_t rb[3] = {64, 64, 128}, bb[3] = {64, 16, 32};
        const void* rp[7]; const void* bp[3];
        static char pool[1 << 16];
        for (int i = 0; i < 7; ++i) rp[i] = pool + 4096 * i;
        for (int i = 0; i < 3; ++i) bp[i] = pool + 32768 + 8192 * i;
        epara_segment seg[7];
        int64_t chunks = 0;
        CHECK(epara_request_segments(rows, off, 3, rb, bb, rp, bp, 1, seg, &chunks) == EPARA_OK && chunks >= 6);
        int64_t per[5];
        int32_t who[23];
        CHECK(epara_dp_deal(7, 23, 5, per, who) == EPARA_OK);
        CHECK(epara_dp_group_count(120, 30) == 4 && epara_inter_request_count(8, 4) == 2 && epara_max_inter_frame_count(100000, 30000) == 3);
    }
    // ---- handler, placement, simulation
    {
        const int32_t N = 6;
        double theo[N], act[N];
        int64_t queued[N];
        for (int i = 0; i < N; ++i) { theo[i] = 10 + i; act[i] = 3 * i; queued[i] = 1000 * i; }
        for (int k = 0; k < 200; ++k) {
            int32_t decision = -1, dest = -1;
            CHECK(epara_handle_request(rnd(0, 100), rnd(0, 100), rnd(0, 1), rnd(0, 3), 2, theo, act, queued, N, rnd(0, N - 1), 2000, 1500, unit(), &decision, &dest) == EPARA_OK);
            CHECK(decision >= 0 && decision <= 4 && dest < N);
        }
        int32_t weights[16], cand[16], out[64], n_out = 0;
        for (int i = 0; i < 16; ++i) { weights[i] = rnd(0, 9); cand[i] = i; }
        CHECK(epara_place_full_models(cand, 16, 0, 0, nullptr, 0, coverage_phi, weights, out, 64, &n_out) == EPARA_OK && n_out <= 16);
        CHECK(epara_place_services(cand, 4, cand, 16, cand + 8, 8, coverage_phi, weights, out, 64, &n_out) == EPARA_OK);
        CHECK(epara_place_full_models(cand, 16, 1, 0, nullptr, 0, coverage_phi, weights, out, 2, &n_out) != EPARA_ERR_NULL);
        const int32_t L = 3, S = 4;
        int64_t c[L * S];
        for (auto& v : c) v = rnd(0, 4) == 0 ? 0 : rnd(500, 4000);
        epara_sim_config cfg = {c, 300, 2000, S, L, 2, 0};
        std::vector<epara_sim_request> reqs(400);
        std::vector<double> draws(reqs.size() * 2);
        for (auto& q : reqs) { q.arrival_us = rnd(0, 200000); q.slo_us = rnd(1000, 20000); q.service = rnd(0, L - 1); q.origin = rnd(0, S - 1); q.frames = rnd(1, 3); q.fps_milli = rnd(0, 2) == 0 ? rnd(1000, 60000) : 0; }
        for (auto& u : draws) u = unit();
        int32_t placements[10];
        for (auto& p : placements) p = rnd(0, L * S - 1);
        epara_sim_result r;
        CHECK(epara_simulate(&cfg, placements, 10, reqs.data(), static_cast<int64_t>(reqs.size()), draws.data(), &r) == EPARA_OK);
        CHECK(r.local + r.timeout + r.offload_exceeded + r.insufficient == static_cast<int64_t>(reqs.size()));
        CHECK(epara_simulate(&cfg, placements, 0, reqs.data(), 5, draws.data(), &r) == EPARA_OK);
    }
    // ---- the oracle's loops and codecs
    {
        const int64_t M = 7, K = 13, N = 5;
        std::vector<double> X(M * K), W(K * N), b(N), Y(M * N), H(M * N);
        for (auto& v : X) v = unit() - 0.5;
        for (auto& v : W) v = unit() - 0.5;
        for (auto& v : b) v = unit();
        for (int act = 0; act < 5; ++act) oracle_dense_forward(X.data(), W.data(), act % 2 ? b.data() : nullptr, M, K, N, 0.5, act, Y.data());
        oracle_dense_forward(X.data(), W.data(), nullptr, 0, K, N, 1.0, 0, Y.data());
        oracle_swiglu_hidden(X.data(), W.data(), W.data(), M, K, N, 1.0, 2.0, H.data());
        std::vector<float> f(300);
        std::vector<uint16_t> h(300);
        std::vector<double> d(300);
        std::vector<uint8_t> q(300);
        for (size_t i = 0; i < f.size(); ++i) f[i] = static_cast<float>((unit() - 0.5) * 1000.0);
        oracle_bf16_encode(f.data(), 300, h.data());
        oracle_bf16_decode(h.data(), 300, d.data());
        oracle_e4m3_encode(d.data(), 300, 1.3, q.data());
        oracle_e4m3_decode(q.data(), 300, 1.3, d.data());
        oracle_act_array(d.data(), 300, 4, d.data());
    }
    std::puts("sanitize_driver: ok");
    return 0;
}
