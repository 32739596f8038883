// Host half of libepara: batch accounting, group planning, visit order, argument helpers.
// Integer-only and deterministic; nothing here touches the GPU.
//
// The planner is the single-GPU part of the allocator of Sec. 3.1: the batching (BS) and
// multi-frame (MF) operators fix how many rows each service's batch has, multi-task (MT)
// puts several services into one launch, and the tile class picked per group is the
// "parallel mode" that group runs in.
#include "epara.h"

#include <algorithm>
#include <climits>
#include <cstring>
#include <functional>
#include <queue>
#include <utility>
#include <vector>

namespace {

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// The cost model of the scheduler (the constants are the header's).
inline int64_t tile_cost(const epara_group_desc& d, const epara_tile& tl, const epara_tile_class* classes, int32_t n_stream_classes)
{
    if (tl.cls >= n_stream_classes) return static_cast<int64_t>(EPARA_COST_PANEL) * d.K;
    const int64_t BM = classes[tl.cls].BM;
    const int64_t units = static_cast<int64_t>(EPARA_COST_PER_COLUMN) * tl.cols * (d.act == EPARA_ACT_SWIGLU ? 2 : 1) +
                          (BM >= 32 ? EPARA_COST_PER_ROW * BM : 0);
    return units * d.K;
}

// Whether the last round of a launch of equal panel tiles is worth cutting along K, and how (see "Splitting K" in
// the header).  n_panel: all tiles of the launch, every one a panel tile of cost `cost` (the class's split_K keeps K
// long enough for every part to hold whole units of four K stages).  Returns the number m of tiles to split (0: none);
// the first m - *n_more of them get *parts parts, the last *n_more one part more.
inline int32_t panel_split_choice(int64_t n_panel, int64_t W, int64_t cost, int32_t* parts, int32_t* n_more)
{
    *parts = 1;
    *n_more = 0;
    const int64_t m = n_panel % W;
    if (n_panel == 0 || m == 0) return 0;
    int64_t best = cost * 9 / 10;                                // must beat 0.9 of a whole tile
    // every tile in P parts
    for (int32_t P = 2; P <= EPARA_SPLIT_MAX_PARTS; ++P) {
        const int64_t t = ((m * P + W - 1) / W) * (cost / P + EPARA_COST_PANEL_PARTIAL);
        if (t < best) { best = t; *parts = P; *n_more = 0; }
    }
    // k parts per workgroup on average: Q = k W parts dealt to the m tiles as evenly as whole numbers allow
    for (int64_t k = 1; k <= EPARA_SPLIT_MAX_PARTS; ++k) {
        const int64_t Q = k * W;
        if (Q < 2 * m || Q > EPARA_SPLIT_MAX_PARTS * m) continue;
        const int64_t base = Q / m, more = Q % m;
        if (more == 0) continue;                                 // the same as every tile in `base` parts
        // the larger parts first, each to the least loaded workgroup (all start level: the whole tiles fill whole rounds)
        std::priority_queue<int64_t, std::vector<int64_t>, std::greater<int64_t>> bins;
        for (int64_t b = 0; b < W; ++b) bins.push(0);
        int64_t t = 0;
        for (int64_t i = 0; i < Q; ++i) {
            const int64_t item = i < (m - more) * base ? cost / base + EPARA_COST_PANEL_PARTIAL : cost / (base + 1) + EPARA_COST_PANEL_PARTIAL;
            const int64_t load = bins.top() + item;
            bins.pop();
            bins.push(load);
            t = std::max(t, load);
        }
        if (t < best) { best = t; *parts = static_cast<int32_t>(base); *n_more = static_cast<int32_t>(more); }
    }
    return *parts > 1 ? static_cast<int32_t>(m) : 0;
}

int32_t check_classes(const epara_tile_class* classes, int32_t n_classes)
{
    if (!classes) return EPARA_ERR_NULL;
    if (n_classes <= 0) return EPARA_ERR_SHAPE;
    for (int32_t c = 0; c < n_classes; ++c) {
        if (classes[c].BM <= 0 || classes[c].BN <= 0 || classes[c].split_K < 0) return EPARA_ERR_SHAPE;
        if (c > 0 && classes[c].max_M <= classes[c - 1].max_M) return EPARA_ERR_SHAPE;
    }
    return EPARA_OK;
}

int32_t class_of(int32_t M, const epara_tile_class* classes, int32_t n_classes)
{
    for (int32_t c = 0; c < n_classes; ++c)
        if (M <= classes[c].max_M) return c;
    return -1;
}

// The panel split of a launch (validated groups and classes): tiles to split, parts.
int32_t panel_split_of(const epara_group_desc* groups, int32_t G, const epara_tile_class* classes, int32_t n_classes,
                       int32_t n_stream_classes, int64_t W, int32_t* parts, int32_t* n_more)
{
    *parts = 1;
    *n_more = 0;
    int32_t cls = -1, K = 0;
    int64_t n = 0;
    for (int32_t g = 0; g < G; ++g) {
        const epara_group_desc& d = groups[g];
        if (d.M <= 0) continue;
        const int32_t c = class_of(d.M, classes, n_classes);
        if (c < n_stream_classes || d.act == EPARA_ACT_SWIGLU) return 0;
        if (cls >= 0 && (c != cls || d.K != K)) return 0;
        if (classes[c].split_K <= 0 || d.K < classes[c].split_K) return 0;
        cls = c; K = d.K;
        n += ceil_div(d.M, classes[c].BM) * ceil_div(d.N, classes[c].BN);
    }
    if (cls < 0 || n > 0xFFFFFF) return 0;
    return panel_split_choice(n, W, static_cast<int64_t>(EPARA_COST_PANEL) * K, parts, n_more);
}

int32_t gated_of(const epara_group_desc* groups, int32_t G, int32_t* gated)
{
    int32_t n_gated = 0, n_live = 0;
    for (int32_t g = 0; g < G; ++g)
        if (groups[g].M > 0) { ++n_live; n_gated += groups[g].act == EPARA_ACT_SWIGLU; }
    if (n_gated != 0 && n_gated != n_live) return EPARA_ERR_DTYPE;
    *gated = n_gated > 0;
    return EPARA_OK;
}


inline int32_t split_parts(const epara_group_desc& d, const epara_tile_class& c) { return c.split_K > 0 && d.K >= c.split_K ? EPARA_SPLIT_PARTS : 1; }

// Cost of one of the `parts` visits of a tile whose whole cost is `cost`: its share of K plus the partial result it leaves.
inline int64_t visit_cost(int64_t cost, int32_t parts, const epara_group_desc& d, const epara_tile& t, const epara_tile_class& c, bool panel = false)
{
    if (parts == 1) return cost;
    if (panel) return cost / parts + EPARA_COST_PANEL_PARTIAL;
    return cost / parts + static_cast<int64_t>(EPARA_COST_PARTIAL) * c.BM * t.cols * (d.act == EPARA_ACT_SWIGLU ? 2 : 1);
}

}  // namespace

extern "C" {

const char* epara_status_string(int32_t status)
{
    switch (status) {
    case EPARA_OK:           return "ok";
    case EPARA_ERR_NULL:     return "required pointer is NULL";
    case EPARA_ERR_SHAPE:    return "bad shape, class table, tile or grid";
    case EPARA_ERR_DTYPE:    return "unsupported dtype or activation";
    case EPARA_ERR_CAPACITY: return "output array too small";
    case EPARA_ERR_ALIGN:    return "pointer or row pitch not 16-byte aligned";
    case EPARA_ERR_HIP:      return "HIP runtime error";
    default:                 return "unknown status";
    }
}

int32_t epara_batch_rows(const int32_t* request_rows, const int64_t* request_off, int32_t G,
                         int32_t* M, int64_t* first_row)
{
    if (G < 0) return EPARA_ERR_SHAPE;
    if (G == 0) return EPARA_OK;
    if (!request_off || !M) return EPARA_ERR_NULL;
    if (request_off[0] < 0) return EPARA_ERR_SHAPE;
    for (int32_t g = 0; g < G; ++g) {
        const int64_t lo = request_off[g], hi = request_off[g + 1];
        if (hi < lo) return EPARA_ERR_SHAPE;
        if (hi > lo && !request_rows) return EPARA_ERR_NULL;
        int64_t acc = 0;
        for (int64_t r = lo; r < hi; ++r) {
            if (request_rows[r] < 0) return EPARA_ERR_SHAPE;
            if (first_row) first_row[r] = acc;
            acc += request_rows[r];
            if (acc > INT32_MAX) return EPARA_ERR_SHAPE;
        }
        M[g] = static_cast<int32_t>(acc);
    }
    return EPARA_OK;
}

int32_t epara_operator_set(int32_t category, int32_t multi_gpu)
{
    int32_t ops;
    if (category == EPARA_CAT_LATENCY)        ops = EPARA_OP_BS | EPARA_OP_MT;
    else if (category == EPARA_CAT_FREQUENCY) ops = EPARA_OP_MF | EPARA_OP_MT | EPARA_OP_BS;
    else return -1;
    if (multi_gpu) ops |= EPARA_OP_MP | (category == EPARA_CAT_FREQUENCY ? EPARA_OP_DP : 0);
    return ops;
}

int64_t epara_max_inter_frame_count(int64_t latency_us, int64_t fps_milli)
{
    if (latency_us < 0 || fps_milli <= 0) return -1;
    const __int128 frames = static_cast<__int128>(latency_us) * fps_milli / 1000000000;
    return frames < 1 ? 1 : static_cast<int64_t>(frames);
}

int32_t epara_dp_deal(int64_t first_frame, int64_t n_frames, int64_t n_groups,
                      int64_t* frames_per_group, int32_t* group_of_frame)
{
    if (n_groups <= 0 || n_groups > INT32_MAX || n_frames < 0 || first_frame < 0) return EPARA_ERR_SHAPE;
    if (frames_per_group) {
        const int64_t base = n_frames / n_groups, extra = n_frames % n_groups, start = first_frame % n_groups;
        for (int64_t g = 0; g < n_groups; ++g)                    // the `extra` groups from `start` on get one more
            frames_per_group[g] = base + (((g - start) % n_groups + n_groups) % n_groups < extra ? 1 : 0);
    }
    if (group_of_frame)
        for (int64_t j = 0; j < n_frames; ++j) group_of_frame[j] = static_cast<int32_t>((first_frame % n_groups + j) % n_groups);
    return EPARA_OK;
}

int32_t epara_handle_request(int64_t now_us, int64_t deadline_us, int32_t local_can_serve,
                             int32_t offload_count, int32_t max_offload,
                             const double* theoretical, const double* actual, const int64_t* queued_us,
                             int32_t n_servers, int32_t self, int64_t sync_delay_us, int64_t slo_us, double u,
                             int32_t* decision, int32_t* destination)
{
    if (!decision || !destination) return EPARA_ERR_NULL;
    *destination = -1;
    if (n_servers <= 0 || self < 0 || self >= n_servers || !(u >= 0.0 && u < 1.0)) return EPARA_ERR_SHAPE;
    if (now_us > deadline_us) { *decision = EPARA_HANDLE_TIMEOUT; return EPARA_OK; }
    if (local_can_serve) { *decision = EPARA_HANDLE_LOCAL; return EPARA_OK; }
    if (offload_count >= max_offload) { *decision = EPARA_HANDLE_OFFLOAD_EXCEEDED; return EPARA_OK; }
    if (!theoretical || !actual || !queued_us) return EPARA_ERR_NULL;
    auto idle = [&](int32_t m) {
        if (m == self || queued_us[m] > sync_delay_us + slo_us) return 0.0;
        const double v = theoretical[m] - actual[m];
        return v > 0.0 ? v : 0.0;
    };
    double total = 0.0;
    for (int32_t m = 0; m < n_servers; ++m) total += idle(m);
    if (!(total > 0.0)) { *decision = EPARA_HANDLE_INSUFFICIENT; return EPARA_OK; }
    double acc = 0.0;
    int32_t last = -1;
    for (int32_t m = 0; m < n_servers; ++m) {
        const double v = idle(m);
        if (v <= 0.0) continue;
        acc += v;
        last = m;
        if (acc > u * total) break;
    }
    *decision = EPARA_HANDLE_OFFLOAD;
    *destination = last;                     // rounding can leave acc == u * total at the end: the last feasible server
    return EPARA_OK;
}

int32_t epara_place_full_models(const int32_t* candidates, int32_t n_candidates, int32_t is_set, int32_t keep_equal,
                                const int32_t* theta0, int32_t n0, epara_phi_fn phi, void* user,
                                int32_t* theta_out, int32_t cap, int32_t* n_out)
{
    if (n_candidates < 0 || n0 < 0 || cap < 0) return EPARA_ERR_SHAPE;
    if (!phi || !n_out || (n_candidates > 0 && !candidates) || (n0 > 0 && !theta0) || (cap > 0 && !theta_out)) return EPARA_ERR_NULL;
    for (int32_t i = 0; i < n_candidates; ++i) if (candidates[i] < 0) return EPARA_ERR_SHAPE;
    for (int32_t i = 0; i < n0; ++i) if (theta0[i] < 0) return EPARA_ERR_SHAPE;
    if (n0 > cap) { *n_out = n0; return EPARA_ERR_CAPACITY; }
    std::vector<int32_t> theta(theta0, theta0 + n0);
    std::vector<char> used(static_cast<size_t>(n_candidates), 0);      // list semantics: chosen positions
    double value = phi(theta.data(), static_cast<int32_t>(theta.size()), user);
    for (;;) {
        int32_t best = -1;
        double best_value = 0.0;
        theta.push_back(0);
        for (int32_t i = 0; i < n_candidates; ++i) {
            if (!is_set && used[i]) continue;
            theta.back() = candidates[i];
            const double v = phi(theta.data(), static_cast<int32_t>(theta.size()), user);
            if (best < 0 || v > best_value) { best = i; best_value = v; }      // ties keep the earliest
        }
        theta.pop_back();
        if (best < 0) break;                                             // no candidate left
        if (!(keep_equal ? best_value >= value : best_value > value)) break;   // this addition is dropped
        if (static_cast<int32_t>(theta.size()) + 1 > cap) { *n_out = static_cast<int32_t>(theta.size()) + 1; return EPARA_ERR_CAPACITY; }
        theta.push_back(candidates[best]);
        used[best] = 1;
        value = best_value;
    }
    *n_out = static_cast<int32_t>(theta.size());
    std::copy(theta.begin(), theta.end(), theta_out);
    return EPARA_OK;
}

int32_t epara_place_services(const int32_t* partial, int32_t n_partial, const int32_t* X, int32_t n_x,
                             const int32_t* X_dot, int32_t n_xdot, epara_phi_fn phi, void* user,
                             int32_t* theta_out, int32_t cap, int32_t* n_out)
{
    if (cap < 0) return EPARA_ERR_SHAPE;
    if (!n_out || (cap > 0 && !theta_out)) return EPARA_ERR_NULL;
    std::vector<int32_t> a(static_cast<size_t>(cap) + 1), b(static_cast<size_t>(cap) + 1);
    int32_t na = 0, nb = 0;
    if (int32_t st = epara_place_full_models(partial, n_partial, 0, 1, nullptr, 0, phi, user, a.data(), cap, &na)) { *n_out = na; return st; }
    if (int32_t st = epara_place_full_models(X, n_x, 1, 0, a.data(), na, phi, user, b.data(), cap, &nb)) { *n_out = nb; return st; }
    if (int32_t st = epara_place_full_models(X_dot, n_xdot, 1, 0, b.data(), nb, phi, user, a.data(), cap, &na)) { *n_out = na; return st; }
    *n_out = na;
    std::copy(a.begin(), a.begin() + na, theta_out);
    return EPARA_OK;
}

int32_t epara_request_segments(const int32_t* request_rows, const int64_t* request_off, int32_t G,
                               const int64_t* request_row_bytes, const int64_t* batch_row_bytes,
                               const void* const* request_ptr, const void* const* batch_ptr, int32_t to_batch,
                               epara_segment* segments, int64_t* n_chunks)
{
    if (G < 0) return EPARA_ERR_SHAPE;
    if (!n_chunks) return EPARA_ERR_NULL;
    *n_chunks = 0;
    if (G == 0) return EPARA_OK;
    if (!request_off || !request_row_bytes || !batch_row_bytes || !batch_ptr) return EPARA_ERR_NULL;
    if (request_off[0] < 0) return EPARA_ERR_SHAPE;
    int64_t chunks = 0;
    for (int32_t g = 0; g < G; ++g) {
        const int64_t lo = request_off[g], hi = request_off[g + 1];
        if (hi < lo || request_row_bytes[g] <= 0 || batch_row_bytes[g] <= 0) return EPARA_ERR_SHAPE;
        if (request_row_bytes[g] % 16 || batch_row_bytes[g] % 16) return EPARA_ERR_ALIGN;
        if (hi > lo && (!request_rows || !request_ptr || !segments)) return EPARA_ERR_NULL;
        int64_t first_row = 0;
        for (int64_t r = lo; r < hi; ++r) {
            if (request_rows[r] < 0) return EPARA_ERR_SHAPE;
            const char* in_batch = static_cast<const char*>(batch_ptr[g]) + first_row * batch_row_bytes[g];
            epara_segment& sg = segments[r];
            sg.src = to_batch ? request_ptr[r] : in_batch;
            sg.dst = const_cast<void*>(to_batch ? static_cast<const void*>(in_batch) : request_ptr[r]);
            sg.bytes = static_cast<int64_t>(request_rows[r]) * (to_batch ? request_row_bytes[g] : batch_row_bytes[g]);
            sg.first_chunk = chunks;
            sg.group = g;
            sg.reserved = 0;
            chunks += ceil_div(sg.bytes, 16384);
            first_row += request_rows[r];
        }
    }
    *n_chunks = chunks;
    return EPARA_OK;
}

int64_t epara_dp_group_count(int64_t rate_required, int64_t rate_of_one_group)
{
    if (rate_required < 0 || rate_of_one_group <= 0) return -1;
    return ceil_div(rate_required, rate_of_one_group);
}

int64_t epara_inter_request_count(int64_t batch_size, int64_t max_inter_frame_count)
{
    if (batch_size < 0 || max_inter_frame_count <= 0) return -1;
    return batch_size / max_inter_frame_count;
}

int32_t epara_compute_table(const double* ms_per_pass, const int32_t* requests_per_pass, int32_t n_services,
                            const double* server_speed, int32_t n_servers, int64_t* compute_us)
{
    if (n_services < 0 || n_servers < 0) return EPARA_ERR_SHAPE;
    if (n_services == 0 || n_servers == 0) return EPARA_OK;
    if (!ms_per_pass || !requests_per_pass || !server_speed || !compute_us) return EPARA_ERR_NULL;
    for (int32_t l = 0; l < n_services; ++l)
        if (!(ms_per_pass[l] > 0.0) || requests_per_pass[l] <= 0) return EPARA_ERR_SHAPE;
    for (int32_t l = 0; l < n_services; ++l)
        for (int32_t n = 0; n < n_servers; ++n) {
            int64_t us = 0;
            if (server_speed[n] > 0.0) {
                const double exact = 1000.0 * ms_per_pass[l] / static_cast<double>(requests_per_pass[l]) / server_speed[n];
                us = static_cast<int64_t>(exact);
                if (static_cast<double>(us) < exact) ++us;
                if (us < 1) us = 1;
            }
            compute_us[static_cast<size_t>(l) * n_servers + n] = us;
        }
    return EPARA_OK;
}

int32_t epara_simulate(const epara_sim_config* config, const int32_t* placements, int32_t n_placements,
                       const epara_sim_request* requests, int64_t n_requests, const double* draws,
                       epara_sim_result* result)
{
    if (!config || !result) return EPARA_ERR_NULL;
    const int32_t N = config->n_servers, L = config->n_services, max_off = config->max_offload;
    const int64_t t = config->sync_delay_us;
    if (N <= 0 || L <= 0 || t <= 0 || max_off < 0 || config->hop_us < 0 || n_placements < 0 || n_requests < 0) return EPARA_ERR_SHAPE;
    if (!config->compute_us || (n_placements > 0 && !placements) || (n_requests > 0 && !requests)) return EPARA_ERR_NULL;
    if (n_requests > 0 && max_off > 0 && !draws) return EPARA_ERR_NULL;
    for (int32_t i = 0; i < n_placements; ++i)
        if (placements[i] < 0 || placements[i] >= static_cast<int64_t>(L) * N) return EPARA_ERR_SHAPE;
    for (int64_t r = 0; r < n_requests; ++r) {
        const epara_sim_request& q = requests[r];
        if (q.service < 0 || q.service >= L || q.origin < 0 || q.origin >= N || q.frames < 1 || q.slo_us < 0 || q.arrival_us < 0 || q.fps_milli < 0)
            return EPARA_ERR_SHAPE;
        for (int32_t k = 0; k < max_off; ++k) {
            const double u = draws[r * max_off + k];
            if (!(u >= 0.0 && u < 1.0)) return EPARA_ERR_SHAPE;
        }
    }

    struct pool {                                            // the instances of one (service, server)
        std::vector<int64_t> free;                           // when each instance is free
        std::vector<std::pair<int64_t, int64_t>> log;        // (decision time, first free time after it)
        std::vector<std::pair<int64_t, int64_t>> done;       // (window index, completions), ascending windows may repeat
    };
    std::vector<pool> pools(static_cast<size_t>(L) * N);
    for (int32_t i = 0; i < n_placements; ++i) pools[placements[i]].free.push_back(0);

    struct event { int64_t time, seq, request; int32_t server, hops; std::vector<int32_t> path; };
    auto later = [](const event& a, const event& b) { return a.time != b.time ? a.time > b.time : a.seq > b.seq; };
    std::priority_queue<event, std::vector<event>, decltype(later)> heap(later);
    for (int64_t r = 0; r < n_requests; ++r) heap.push({requests[r].arrival_us, r, r, requests[r].origin, 0, {requests[r].origin}});
    int64_t seq = n_requests;

    epara_sim_result out;
    std::memset(&out, 0, sizeof out);
    std::vector<double> theoretical(N), actual(N);
    std::vector<int64_t> queued(N);
    while (!heap.empty()) {
        event e = heap.top();
        heap.pop();
        const epara_sim_request& q = requests[e.request];
        const int32_t l = q.service, n = e.server;
        const int64_t now = e.time, deadline = q.arrival_us + q.slo_us;
        pool& here = pools[static_cast<size_t>(l) * N + n];
        const int64_t c_here = config->compute_us[static_cast<size_t>(l) * N + n];
        int32_t slot = -1, local_ok = 0;
        int64_t finish = 0;
        if (!here.free.empty() && c_here > 0) {
            slot = 0;
            for (size_t i = 1; i < here.free.size(); ++i)
                if (here.free[i] < here.free[slot]) slot = static_cast<int32_t>(i);
            finish = std::max(now, here.free[slot]) + q.frames * c_here;
            local_ok = finish <= deadline || q.fps_milli > 0;    // a stream is taken at whatever rate the instance gives
        }
        const int64_t J = now / t - 1;
        for (int32_t m = 0; m < N; ++m) {
            theoretical[m] = actual[m] = 0.0;
            queued[m] = 0;
            const pool& there = pools[static_cast<size_t>(l) * N + m];
            const int64_t c = config->compute_us[static_cast<size_t>(l) * N + m];
            if (there.free.empty() || c <= 0 || std::find(e.path.begin(), e.path.end(), m) != e.path.end()) continue;
            theoretical[m] = static_cast<double>(there.free.size()) * 1e6 / static_cast<double>(c);
            if (J >= 1) {
                int64_t completions = 0;
                for (const auto& d : there.done)
                    if (d.first == J) completions += d.second;
                actual[m] = static_cast<double>(completions) * 1e6 / static_cast<double>(t);
                int64_t first_free = 0;
                for (const auto& g : there.log)
                    if (g.first <= J * t) first_free = g.second;
                queued[m] = std::max<int64_t>(0, first_free - J * t);
            }
        }
        const double u = e.hops < max_off ? draws[e.request * max_off + e.hops] : 0.0;
        int32_t decision = 0, dest = -1;
        if (int32_t st = epara_handle_request(now, deadline, local_ok, e.hops, max_off, theoretical.data(), actual.data(),
                                              queued.data(), N, n, t, q.slo_us, u, &decision, &dest)) return st;
        switch (decision) {
        case EPARA_HANDLE_LOCAL: {
            here.free[slot] = finish;
            here.log.push_back({now, *std::min_element(here.free.begin(), here.free.end())});
            here.done.push_back({(finish + t - 1) / t, 1});
            ++out.local;
            if (q.fps_milli > 0) {                               // frames count, in proportion to the achieved rate
                const double achieved = static_cast<double>(q.frames) * 1e6 / static_cast<double>(finish - q.arrival_us);
                const double share = achieved / (static_cast<double>(q.fps_milli) / 1000.0);
                out.satisfied += static_cast<double>(q.frames) * (share < 1.0 ? share : 1.0);
            } else {
                out.satisfied += 1.0;
            }
            break;
        }
        case EPARA_HANDLE_OFFLOAD: {
            ++out.offloaded;
            event f{now + config->hop_us, seq++, e.request, dest, e.hops + 1, e.path};
            f.path.push_back(dest);
            heap.push(std::move(f));
            break;
        }
        case EPARA_HANDLE_TIMEOUT: ++out.timeout; break;
        case EPARA_HANDLE_OFFLOAD_EXCEEDED: ++out.offload_exceeded; break;
        default: ++out.insufficient; break;
        }
    }
    *result = out;
    return EPARA_OK;
}

int32_t epara_plan_groups(const epara_group_desc* groups, int32_t G,
                          const epara_tile_class* classes, int32_t n_classes,
                          int64_t* row_off, int64_t* x_off, int64_t* y_off,
                          epara_tile* tiles, int64_t tiles_cap, int64_t* n_tiles)
{
    if (G < 0) return EPARA_ERR_SHAPE;
    if (!n_tiles || (G > 0 && !groups)) return EPARA_ERR_NULL;
    if (int32_t st = check_classes(classes, n_classes)) return st;

    // pass 1: validate and count, so that nothing is written on a shape error
    int64_t need = 0;
    for (int32_t g = 0; g < G; ++g) {
        const epara_group_desc& d = groups[g];
        if (d.M < 0 || d.K <= 0 || d.N <= 0) return EPARA_ERR_SHAPE;
        if (d.M == 0) continue;
        const int32_t c = class_of(d.M, classes, n_classes);
        if (c < 0) return EPARA_ERR_SHAPE;
        need += ceil_div(d.M, classes[c].BM) * ceil_div(d.N, classes[c].BN);
    }
    *n_tiles = need;

    int64_t rows = 0, xs = 0, ys = 0;
    for (int32_t g = 0; g <= G; ++g) {
        if (row_off) row_off[g] = rows;
        if (x_off) x_off[g] = xs;
        if (y_off) y_off[g] = ys;
        if (g == G) break;
        rows += groups[g].M;
        xs += static_cast<int64_t>(groups[g].M) * groups[g].K;
        ys += static_cast<int64_t>(groups[g].M) * groups[g].N;
    }
    if (!tiles) return EPARA_OK;
    if (tiles_cap < need) return EPARA_ERR_CAPACITY;

    epara_tile* out = tiles;
    for (int32_t g = 0; g < G; ++g) {
        const epara_group_desc& d = groups[g];
        if (d.M == 0) continue;
        const int32_t c = class_of(d.M, classes, n_classes);
        const int32_t BM = classes[c].BM, BN = classes[c].BN;
        for (int64_t m0 = 0; m0 < d.M; m0 += BM)
            for (int64_t n0 = 0; n0 < d.N; n0 += BN) {
                out->group = g;
                out->m0 = static_cast<int32_t>(m0);
                out->n0 = static_cast<int32_t>(n0);
                out->rows = static_cast<int32_t>(std::min<int64_t>(BM, d.M - m0));
                out->cols = static_cast<int32_t>(std::min<int64_t>(BN, d.N - n0));
                out->cls = c;
                ++out;
            }
    }
    return EPARA_OK;
}

int32_t epara_schedule_chain(epara_phase_schedule* phases, int32_t n_phases,
                             int32_t n_workgroups, int32_t n_xcd, int32_t panel_m, int32_t panel_n)
{
    if (n_phases < 0) return EPARA_ERR_SHAPE;
    if (n_phases > 0 && !phases) return EPARA_ERR_NULL;
    if (n_workgroups <= 0 || n_xcd <= 0 || n_workgroups % n_xcd != 0 || panel_m <= 0 || panel_n <= 0)
        return EPARA_ERR_SHAPE;
    const int64_t W = n_workgroups, X = n_xcd, per_die = W / X;

    // per phase: where each group's tiles start in the canonical table, and which class it was cut with
    std::vector<std::vector<int64_t>> first(static_cast<size_t>(n_phases));
    std::vector<std::vector<int32_t>> cls(static_cast<size_t>(n_phases));
    for (int32_t p = 0; p < n_phases; ++p) {
        const epara_phase_schedule& ph = phases[p];
        if (ph.G < 0 || ph.n_tiles < 0) return EPARA_ERR_SHAPE;
        if ((ph.G > 0 && !ph.groups) || (ph.n_tiles > 0 && !ph.tiles)) return EPARA_ERR_NULL;
        if (int32_t st = check_classes(ph.classes, ph.n_classes)) return st;
        if (ph.n_stream_classes < 0 || ph.n_stream_classes > ph.n_classes) return EPARA_ERR_SHAPE;
        if (ph.n_tiles > INT32_MAX) return EPARA_ERR_SHAPE;
        first[p].assign(static_cast<size_t>(ph.G), -1);
        cls[p].assign(static_cast<size_t>(ph.G), -1);
        for (int64_t t = 0; t < ph.n_tiles; ++t) {
            const epara_tile& tl = ph.tiles[t];
            if (tl.group < 0 || tl.group >= ph.G || tl.cls < 0 || tl.cls >= ph.n_classes) return EPARA_ERR_SHAPE;
            if (first[p][tl.group] < 0) { first[p][tl.group] = t; cls[p][tl.group] = tl.cls; }
            else if (cls[p][tl.group] != tl.cls) return EPARA_ERR_SHAPE;
        }
        // every group's tile count must be what the grid rule gives, or the table is not canonical
        int64_t expect = 0;
        for (int32_t g = 0; g < ph.G; ++g)
            if (first[p][g] >= 0) {
                if (first[p][g] != expect) return EPARA_ERR_SHAPE;
                expect += ceil_div(ph.groups[g].M, ph.classes[cls[p][g]].BM) * ceil_div(ph.groups[g].N, ph.classes[cls[p][g]].BN);
            }
        if (expect != ph.n_tiles) return EPARA_ERR_SHAPE;
    }

    std::vector<std::vector<std::vector<int32_t>>> lists(static_cast<size_t>(n_phases),
                                                          std::vector<std::vector<int32_t>>(static_cast<size_t>(W)));
    std::vector<int64_t> load(static_cast<size_t>(W), 0);

    // 1. panel tiles, phase after phase, each to the least loaded workgroup; among equally loaded ones the
    // die-major rank decides (rank r = workgroup (r mod per_die) * X + r div per_die), so that tiles of equal
    // cost go round robin and the per_die tiles that run together on one die are consecutive in the sequence
    typedef std::pair<int64_t, int64_t> ranked;                 // (load, rank): smallest first
    std::priority_queue<ranked, std::vector<ranked>, std::greater<ranked>> panel_heap;
    for (int64_t r = 0; r < W; ++r) panel_heap.push({0, r});
    std::vector<int32_t> class_order, members;
    // a single launch of equal panel tiles may visit the tiles of its last round in parts of K
    int32_t panel_parts = 1, panel_more = 0;
    const int64_t n_panel_split = n_phases == 1 ? panel_split_of(phases[0].groups, phases[0].G, phases[0].classes, phases[0].n_classes,
                                                                 phases[0].n_stream_classes, W, &panel_parts, &panel_more) : 0;
    for (int32_t p = 0; p < n_phases; ++p) {
        const epara_phase_schedule& ph = phases[p];
        class_order.clear();
        for (int32_t c = ph.n_stream_classes; c < ph.n_classes; ++c) class_order.push_back(c);
        std::stable_sort(class_order.begin(), class_order.end(), [&](int32_t a, int32_t b) {
            return static_cast<int64_t>(ph.classes[a].BM) * ph.classes[a].BN > static_cast<int64_t>(ph.classes[b].BM) * ph.classes[b].BN;
        });
        for (int32_t c : class_order) {
            members.clear();
            for (int32_t g = 0; g < ph.G; ++g)
                if (cls[p][g] == c) members.push_back(g);
            std::stable_sort(members.begin(), members.end(),
                             [&](int32_t a, int32_t b) { return ph.groups[a].K > ph.groups[b].K; });
            const int64_t BM = ph.classes[c].BM, BN = ph.classes[c].BN;
            for (int32_t g : members) {
                const int64_t TM = ceil_div(ph.groups[g].M, BM), TN = ceil_div(ph.groups[g].N, BN);
                for (int64_t pn = 0; pn < TN; pn += panel_n)
                    for (int64_t pm = 0; pm < TM; pm += panel_m)
                        for (int64_t tn = pn; tn < std::min<int64_t>(pn + panel_n, TN); ++tn)
                            for (int64_t tm = pm; tm < std::min<int64_t>(pm + panel_m, TM); ++tm) {
                                const int64_t tile = first[p][g] + tm * TN + tn;
                                if (tile >= ph.n_tiles - n_panel_split) continue;      // visited in parts, after the whole tiles
                                const ranked top = panel_heap.top();
                                panel_heap.pop();
                                const int64_t x = top.second / per_die, i = top.second % per_die, b = i * X + x;
                                lists[p][b].push_back(static_cast<int32_t>(tile));
                                load[b] += static_cast<int64_t>(EPARA_COST_PANEL) * ph.groups[g].K;
                                panel_heap.push({load[b], top.second});
                            }
            }
        }
    }

    if (n_panel_split > 0) {                                     // the parts: tile by tile, part by part, same rule
        const epara_phase_schedule& ph = phases[0];
        for (int64_t tile = ph.n_tiles - n_panel_split; tile < ph.n_tiles; ++tile) {
            const int32_t P = panel_parts + (tile >= ph.n_tiles - panel_more ? 1 : 0);       // the last panel_more tiles: one part more
            const int64_t each = static_cast<int64_t>(EPARA_COST_PANEL) * ph.groups[ph.tiles[tile].group].K / P + EPARA_COST_PANEL_PARTIAL;
            for (int32_t j = 0; j < P; ++j) {
                const ranked top = panel_heap.top();
                panel_heap.pop();
                const int64_t x = top.second / per_die, i = top.second % per_die, b = i * X + x;
                lists[0][b].push_back(EPARA_ORDER_ENTRY(static_cast<int32_t>(tile), j, P));
                load[b] += each;
                panel_heap.push({load[b], top.second});
            }
        }
    }

    // 2. streaming tiles of every phase together, longest first onto the least loaded workgroup
    struct item { int64_t cost; int32_t phase; int32_t tile; };
    std::vector<item> stream;
    for (int32_t p = 0; p < n_phases; ++p) {
        const epara_phase_schedule& ph = phases[p];
        for (int64_t t = 0; t < ph.n_tiles; ++t)
            if (ph.tiles[t].cls < ph.n_stream_classes) {
                const epara_group_desc& d = ph.groups[ph.tiles[t].group];
                const epara_tile_class& c = ph.classes[ph.tiles[t].cls];
                const int64_t cost = tile_cost(d, ph.tiles[t], ph.classes, ph.n_stream_classes);
                const int32_t parts = n_phases == 1 ? split_parts(d, c) : 1;       // the phases of a chain are not split
                if (parts == 1) { stream.push_back({cost, p, static_cast<int32_t>(t)}); continue; }
                if (ph.n_tiles > 0xFFFFFF) return EPARA_ERR_SHAPE;
                const int64_t each = visit_cost(cost, parts, d, ph.tiles[t], c);
                for (int32_t j = 0; j < parts; ++j) stream.push_back({each, p, EPARA_ORDER_ENTRY(static_cast<int32_t>(t), j, parts)});
            }
    }
    std::stable_sort(stream.begin(), stream.end(), [](const item& a, const item& b) { return a.cost > b.cost; });
    typedef std::pair<int64_t, int32_t> entry;                  // (load, workgroup): smallest first
    std::priority_queue<entry, std::vector<entry>, std::greater<entry>> heap;
    for (int32_t b = 0; b < W; ++b) heap.push({load[b], b});
    for (const item& it : stream) {
        entry e = heap.top();
        heap.pop();
        lists[it.phase][e.second].push_back(it.tile);
        heap.push({e.first + it.cost, e.second});
    }

    int32_t status = EPARA_OK;
    for (int32_t p = 0; p < n_phases; ++p) {
        epara_phase_schedule& ph = phases[p];
        size_t longest = 0, total = 0;
        for (const auto& v : lists[p]) { longest = std::max(longest, v.size()); total += v.size(); }
        if (static_cast<int64_t>(total) < ph.n_tiles) return EPARA_ERR_SHAPE;
        ph.n_slots = static_cast<int64_t>(longest) * W;
        if (!ph.order) continue;
        if (ph.order_cap < ph.n_slots) { status = EPARA_ERR_CAPACITY; continue; }
        std::fill(ph.order, ph.order + ph.n_slots, -1);
        for (int64_t b = 0; b < W; ++b)
            for (size_t j = 0; j < lists[p][b].size(); ++j) ph.order[static_cast<int64_t>(j) * W + b] = lists[p][b][j];
    }
    return status;
}

int32_t epara_schedule_tiles(const epara_group_desc* groups, int32_t G,
                             const epara_tile_class* classes, int32_t n_classes, int32_t n_stream_classes,
                             const epara_tile* tiles, int64_t n_tiles,
                             int32_t n_workgroups, int32_t n_xcd, int32_t panel_m, int32_t panel_n,
                             int32_t* order, int64_t order_cap, int64_t* n_slots)
{
    if (G < 0 || n_tiles < 0) return EPARA_ERR_SHAPE;
    if (!n_slots || (G > 0 && !groups) || (n_tiles > 0 && !tiles)) return EPARA_ERR_NULL;
    epara_phase_schedule ph;
    std::memset(&ph, 0, sizeof ph);
    ph.groups = groups; ph.classes = classes; ph.tiles = tiles; ph.order = order;
    ph.n_tiles = n_tiles; ph.order_cap = order_cap;
    ph.G = G; ph.n_classes = n_classes; ph.n_stream_classes = n_stream_classes;
    const int32_t st = epara_schedule_chain(&ph, 1, n_workgroups, n_xcd, panel_m, panel_n);
    if (st == EPARA_OK || st == EPARA_ERR_CAPACITY) *n_slots = ph.n_slots;
    return st;
}

namespace {

// One candidate of a phase: a class table and the canonical tiles it gives.
struct phase_option {
    epara_tile_class classes[4];
    int32_t n_classes = 0, n_stream = 0, narrow = 0;
    std::vector<epara_tile> tiles;
};

int32_t phase_options(const epara_group_desc* groups, int32_t G, int32_t in_dtype, std::vector<phase_option>& out)
{
    if (G < 0) return EPARA_ERR_SHAPE;
    if (G > 0 && !groups) return EPARA_ERR_NULL;
    int32_t gated = 0;
    if (int32_t st = gated_of(groups, G, &gated)) return st;
    int32_t max_M = 0;
    for (int32_t g = 0; g < G; ++g) max_M = std::max(max_M, groups[g].M);
    const int n_opt = (in_dtype != EPARA_F32 && max_M > 32) ? 2 : 1;
    out.resize(static_cast<size_t>(n_opt));
    for (int narrow = 0; narrow < n_opt; ++narrow) {
        phase_option& o = out[narrow];
        o.narrow = narrow;
        if (int32_t st = epara_kernel_classes(in_dtype, gated, narrow, o.classes, 4, &o.n_classes, &o.n_stream)) return st;
        int64_t n = 0;
        if (int32_t st = epara_plan_groups(groups, G, o.classes, o.n_classes, nullptr, nullptr, nullptr, nullptr, 0, &n)) return st;
        o.tiles.resize(static_cast<size_t>(n));
        if (int32_t st = epara_plan_groups(groups, G, o.classes, o.n_classes, nullptr, nullptr, nullptr, o.tiles.data(), n, &n)) return st;
    }
    return EPARA_OK;
}

void fill_plan(epara_launch_plan& plan, const phase_option& o, int32_t gated, int64_t n_slots, int64_t makespan)
{
    std::memset(&plan, 0, sizeof plan);
    std::memcpy(plan.classes, o.classes, sizeof(epara_tile_class) * o.n_classes);
    plan.n_classes = o.n_classes; plan.n_stream_classes = o.n_stream; plan.narrow = o.narrow; plan.gated = gated;
    plan.n_tiles = static_cast<int64_t>(o.tiles.size()); plan.n_slots = n_slots; plan.makespan = makespan;
}

}  // namespace

int32_t epara_plan_chain(epara_chain_plan_phase* phases, int32_t n_phases, int32_t in_dtype,
                         int32_t n_workgroups, int32_t n_xcd, int32_t panel_m, int32_t panel_n, int64_t* finish)
{
    if (n_phases < 1 || n_phases > EPARA_MAX_CHAIN_PHASES) return EPARA_ERR_SHAPE;
    if (!phases) return EPARA_ERR_NULL;
    if (n_workgroups <= 0 || n_xcd <= 0 || n_workgroups % n_xcd != 0 || panel_m <= 0 || panel_n <= 0) return EPARA_ERR_SHAPE;
    const int64_t W = n_workgroups;
    std::vector<std::vector<phase_option>> options(static_cast<size_t>(n_phases));
    std::vector<int32_t> gated(static_cast<size_t>(n_phases), 0);
    for (int32_t p = 0; p < n_phases; ++p) {
        if (int32_t st = phase_options(phases[p].groups, phases[p].G, in_dtype, options[p])) return st;
        gated_of(phases[p].groups, phases[p].G, &gated[p]);
        if (phases[p].producer) {
            if (p == 0) return EPARA_ERR_SHAPE;
            for (int32_t g = 0; g < phases[p].G; ++g)
                if (phases[p].producer[g] < -1 || phases[p].producer[g] >= phases[p - 1].G) return EPARA_ERR_SHAPE;
        }
    }
    // every combination, first phase varying slowest, wide before narrow
    int64_t best_finish = -1;
    std::vector<int> best_pick;
    std::vector<std::vector<int32_t>> best_order;
    std::vector<int> pick(static_cast<size_t>(n_phases), 0);
    for (;;) {
        std::vector<epara_phase_schedule> sched(static_cast<size_t>(n_phases));
        std::vector<std::vector<int32_t>> order(static_cast<size_t>(n_phases));
        for (int pass = 0; pass < 2; ++pass) {
            for (int32_t p = 0; p < n_phases; ++p) {
                const phase_option& o = options[p][pick[p]];
                epara_phase_schedule& ph = sched[p];
                if (pass == 0) {
                    std::memset(&ph, 0, sizeof ph);
                    ph.groups = phases[p].groups; ph.classes = o.classes; ph.tiles = o.tiles.data();
                    ph.n_tiles = static_cast<int64_t>(o.tiles.size());
                    ph.G = phases[p].G; ph.n_classes = o.n_classes; ph.n_stream_classes = o.n_stream;
                } else {
                    order[p].assign(static_cast<size_t>(ph.n_slots), -1);
                    ph.order = order[p].data(); ph.order_cap = ph.n_slots;
                }
            }
            if (int32_t st = epara_schedule_chain(sched.data(), n_phases, n_workgroups, n_xcd, panel_m, panel_n)) return st;
        }
        // replay under the cost model, waits included
        std::vector<int64_t> clock(static_cast<size_t>(W), 0), ready_prev;
        for (int32_t p = 0; p < n_phases; ++p) {
            const phase_option& o = options[p][pick[p]];
            std::vector<int64_t> ready(static_cast<size_t>(phases[p].G), 0);
            const int64_t rows = sched[p].n_slots / W;
            for (int64_t j = 0; j < rows; ++j)
                for (int64_t b = 0; b < W; ++b) {
                    const int32_t e = order[p][static_cast<size_t>(j * W + b)];
                    if (e < 0) continue;
                    const epara_tile& tl = o.tiles[EPARA_ORDER_TILE(e)];
                    int64_t start = clock[b];
                    if (p > 0 && phases[p].producer && phases[p].producer[tl.group] >= 0)
                        start = std::max(start, ready_prev[phases[p].producer[tl.group]]);
                    clock[b] = start + visit_cost(tile_cost(phases[p].groups[tl.group], tl, o.classes, o.n_stream), (e >> 28) + 1,
                                                  phases[p].groups[tl.group], tl, o.classes[tl.cls], tl.cls >= o.n_stream);
                    ready[tl.group] = std::max(ready[tl.group], clock[b]);
                }
            ready_prev.swap(ready);
        }
        const int64_t fin = *std::max_element(clock.begin(), clock.end());
        if (best_finish < 0 || fin < best_finish) { best_finish = fin; best_pick = pick; best_order = order; }
        int32_t p = n_phases - 1;
        while (p >= 0 && ++pick[p] == static_cast<int>(options[p].size())) pick[p--] = 0;
        if (p < 0) break;
    }
    if (finish) *finish = best_finish;
    int32_t status = EPARA_OK, base = 0;
    for (int32_t p = 0; p < n_phases; ++p) {
        const phase_option& o = options[p][best_pick[p]];
        epara_chain_plan_phase& ph = phases[p];
        // a phase's own makespan: its workgroups' costs in this phase alone
        std::vector<int64_t> load(static_cast<size_t>(W), 0);
        for (size_t i = 0; i < best_order[p].size(); ++i)
            if (best_order[p][i] >= 0) {
                const int32_t e = best_order[p][i];
                const epara_tile& tl = o.tiles[EPARA_ORDER_TILE(e)];
                load[i % W] += visit_cost(tile_cost(ph.groups[tl.group], tl, o.classes, o.n_stream), (e >> 28) + 1, ph.groups[tl.group], tl,
                                          o.classes[tl.cls], tl.cls >= o.n_stream);
            }
        fill_plan(ph.plan, o, gated[p], static_cast<int64_t>(best_order[p].size()), *std::max_element(load.begin(), load.end()));
        ph.counter_base = base;
        base += ph.G;
        if (ph.tiles) {
            if (ph.tiles_cap < ph.plan.n_tiles) status = EPARA_ERR_CAPACITY;
            else std::copy(o.tiles.begin(), o.tiles.end(), ph.tiles);
        }
        if (ph.order) {
            if (ph.order_cap < ph.plan.n_slots) status = EPARA_ERR_CAPACITY;
            else std::copy(best_order[p].begin(), best_order[p].end(), ph.order);
        }
    }
    if (status != EPARA_OK) return status;
    for (int32_t p = 1; p < n_phases; ++p) {
        epara_chain_plan_phase& ph = phases[p];
        if (!ph.producer || !ph.waits) continue;
        const phase_option& prev = options[p - 1][best_pick[p - 1]];
        if (int32_t st = epara_chain_waits(prev.tiles.data(), static_cast<int64_t>(prev.tiles.size()), phases[p - 1].G,
                                           phases[p - 1].counter_base, ph.producer, ph.G, ph.waits)) return st;
    }
    return EPARA_OK;
}

int32_t epara_plan_launch(const epara_group_desc* groups, int32_t G, int32_t in_dtype,
                          int32_t n_workgroups, int32_t n_xcd, int32_t panel_m, int32_t panel_n,
                          int64_t* row_off, int64_t* x_off, int64_t* y_off,
                          epara_tile* tiles, int64_t tiles_cap, int32_t* order, int64_t order_cap,
                          int32_t* split_base, epara_launch_plan* plan)
{
    if (!plan) return EPARA_ERR_NULL;
    epara_chain_plan_phase ph;
    std::memset(&ph, 0, sizeof ph);
    ph.groups = groups; ph.G = G; ph.tiles = tiles; ph.tiles_cap = tiles_cap; ph.order = order; ph.order_cap = order_cap;
    const int32_t st = epara_plan_chain(&ph, 1, in_dtype, n_workgroups, n_xcd, panel_m, panel_n, nullptr);
    if (st != EPARA_OK && st != EPARA_ERR_CAPACITY) return st;
    *plan = ph.plan;
    if (int32_t s3 = epara_split_layout(groups, G, plan->classes, plan->n_classes, plan->n_stream_classes, split_base,
                                        &plan->n_split_tiles, &plan->workspace_bytes)) return s3;
    int32_t panel_parts = 1, panel_more = 0;
    plan->n_panel_split_tiles = panel_split_of(groups, G, plan->classes, plan->n_classes, plan->n_stream_classes, n_workgroups, &panel_parts, &panel_more);
    plan->workspace_bytes = epara_split_workspace_bytes(plan->n_split_tiles, plan->n_panel_split_tiles);
    if (row_off || x_off || y_off) {
        int64_t n = 0;
        if (int32_t s2 = epara_plan_groups(groups, G, plan->classes, plan->n_classes, row_off, x_off, y_off, nullptr, 0, &n)) return s2;
    }
    return st;
}

int32_t epara_chain_waits(const epara_tile* producer_tiles, int64_t n_producer_tiles, int32_t G_producer,
                          int32_t counter_base, const int32_t* producer, int32_t G_consumer,
                          epara_chain_wait* waits)
{
    if (n_producer_tiles < 0 || G_producer < 0 || G_consumer < 0 || counter_base < 0) return EPARA_ERR_SHAPE;
    if ((n_producer_tiles > 0 && !producer_tiles) || (G_consumer > 0 && (!producer || !waits))) return EPARA_ERR_NULL;
    std::vector<int64_t> count(static_cast<size_t>(G_producer), 0);
    for (int64_t t = 0; t < n_producer_tiles; ++t) {
        const int32_t g = producer_tiles[t].group;
        if (g < 0 || g >= G_producer) return EPARA_ERR_SHAPE;
        ++count[g];
    }
    for (int32_t g = 0; g < G_consumer; ++g)
        if (producer[g] >= G_producer || producer[g] < -1) return EPARA_ERR_SHAPE;
    for (int32_t g = 0; g < G_consumer; ++g) {
        const int32_t q = producer[g];
        waits[g].counter = q < 0 ? -1 : counter_base + q;
        waits[g].need = q < 0 ? 0 : static_cast<int32_t>(count[q]);
    }
    return EPARA_OK;
}

int32_t epara_split_layout(const epara_group_desc* groups, int32_t G,
                           const epara_tile_class* classes, int32_t n_classes, int32_t n_stream_classes,
                           int32_t* split_base, int32_t* n_split_tiles, int64_t* workspace_bytes)
{
    if (G < 0) return EPARA_ERR_SHAPE;
    if (!n_split_tiles || !workspace_bytes || (G > 0 && !groups)) return EPARA_ERR_NULL;
    if (int32_t st = check_classes(classes, n_classes)) return st;
    if (n_stream_classes < 0 || n_stream_classes > n_classes) return EPARA_ERR_SHAPE;
    int64_t n = 0;
    for (int32_t g = 0; g < G; ++g) {
        const epara_group_desc& d = groups[g];
        if (d.M < 0 || d.K <= 0 || d.N <= 0) return EPARA_ERR_SHAPE;
        int32_t base = -1;
        if (d.M > 0) {
            const int32_t c = class_of(d.M, classes, n_classes);
            if (c < 0) return EPARA_ERR_SHAPE;
            if (c < n_stream_classes && split_parts(d, classes[c]) > 1) {
                base = static_cast<int32_t>(n);
                n += ceil_div(d.M, classes[c].BM) * ceil_div(d.N, classes[c].BN);
            }
        }
        if (split_base) split_base[g] = base;
    }
    if (n > 0xFFFFFF) return EPARA_ERR_SHAPE;
    *n_split_tiles = static_cast<int32_t>(n);
    *workspace_bytes = epara_split_workspace_bytes(static_cast<int32_t>(n), 0);
    return EPARA_OK;
}

int64_t epara_split_workspace_bytes(int32_t n_split_tiles, int32_t n_panel_split_tiles)
{
    if (n_split_tiles < 0 || n_panel_split_tiles < 0) return -1;
    const int64_t n = static_cast<int64_t>(n_split_tiles) + n_panel_split_tiles;
    if (n == 0) return 0;
    return (n * 4 + 255) / 256 * 256 + static_cast<int64_t>(n_split_tiles) * EPARA_SPLIT_MAX_PARTS * EPARA_SPLIT_STRIDE +
           static_cast<int64_t>(n_panel_split_tiles) * EPARA_SPLIT_MAX_PARTS * EPARA_PANEL_SPLIT_STRIDE;
}

int32_t epara_panel_split(const epara_group_desc* groups, int32_t G,
                          const epara_tile_class* classes, int32_t n_classes, int32_t n_stream_classes,
                          int32_t n_workgroups, int32_t* n_panel_split_tiles, int32_t* parts, int32_t* n_more)
{
    if (G < 0 || n_workgroups <= 0) return EPARA_ERR_SHAPE;
    if (!n_panel_split_tiles || !parts || !n_more || (G > 0 && !groups)) return EPARA_ERR_NULL;
    if (int32_t st = check_classes(classes, n_classes)) return st;
    if (n_stream_classes < 0 || n_stream_classes > n_classes) return EPARA_ERR_SHAPE;
    for (int32_t g = 0; g < G; ++g) {
        if (groups[g].M < 0 || groups[g].K <= 0 || groups[g].N <= 0) return EPARA_ERR_SHAPE;
        if (groups[g].M > 0 && class_of(groups[g].M, classes, n_classes) < 0) return EPARA_ERR_SHAPE;
    }
    *n_panel_split_tiles = panel_split_of(groups, G, classes, n_classes, n_stream_classes, n_workgroups, parts, n_more);
    return EPARA_OK;
}

int64_t epara_workspace_bytes(const epara_group_desc* groups, int32_t G, int32_t in_dtype, int32_t n_workgroups)
{
    if (G < 0 || n_workgroups <= 0 || (in_dtype != EPARA_F32 && in_dtype != EPARA_BF16 && in_dtype != EPARA_FP8_E4M3)) return -1;
    if (G > 0 && !groups) return -1;
    if (in_dtype == EPARA_F32) return 0;
    int32_t gated = 0;
    if (gated_of(groups, G, &gated) != EPARA_OK) return -1;
    int64_t worst = 0;
    for (int narrow = 0; narrow < 2; ++narrow) {
        epara_tile_class classes[4];
        int32_t nc = 0, ns = 0, n_split = 0;
        int64_t bytes = 0;
        if (epara_kernel_classes(in_dtype, gated, narrow, classes, 4, &nc, &ns) != EPARA_OK) return -1;
        if (epara_split_layout(groups, G, classes, nc, ns, nullptr, &n_split, &bytes) != EPARA_OK) return -1;
        int32_t parts = 1, more = 0;
        const int32_t n_panel = panel_split_of(groups, G, classes, nc, ns, n_workgroups, &parts, &more);
        worst = std::max(worst, epara_split_workspace_bytes(n_split, n_panel));
    }
    return worst;
}

int32_t epara_kernel_classes(int32_t in_dtype, int32_t gated, int32_t narrow,
                             epara_tile_class* classes, int32_t cap, int32_t* n_classes,
                             int32_t* n_stream_classes)
{
    if (!n_classes || !n_stream_classes) return EPARA_ERR_NULL;
    epara_tile_class table[4];
    int32_t n = 0, ns = 0;
    if (in_dtype == EPARA_F32) {
        if (gated) return EPARA_ERR_DTYPE;
        table[n++] = {16, 16, 64, 0};       // K split over the four waves of a workgroup
        table[n++] = {INT32_MAX, 64, 64, 0};
    } else if (in_dtype == EPARA_BF16 || in_dtype == EPARA_FP8_E4M3) {
        // weight-streaming classes: the whole batch (1, 2 or 4 blocks of 16 rows) against 2, 4 or 8
        // weight column blocks, so that activations re-read per weight byte stay constant
        const int32_t split_K = in_dtype == EPARA_BF16 ? EPARA_SPLIT_K_BF16 : 0;   // where two visits pay (measured)
        table[n++] = {16, 16, gated ? 16 : 32, 0};
        table[n++] = {32, 32, gated ? 32 : 64, split_K};
        table[n++] = {64, 64, (gated ? 64 : 128) >> (narrow ? 1 : 0), split_K};
        ns = 3;
        table[n++] = {INT32_MAX, 256, gated ? 128 : 256, (gated || in_dtype != EPARA_BF16) ? 0 : EPARA_PANEL_SPLIT_K};  // matrix-core class
    } else {
        return EPARA_ERR_DTYPE;
    }
    *n_classes = n;
    *n_stream_classes = ns;
    if (!classes) return EPARA_OK;
    if (cap < n) return EPARA_ERR_CAPACITY;
    std::memcpy(classes, table, sizeof(epara_tile_class) * n);
    return EPARA_OK;
}

int32_t epara_ffn_swiglu_args(const epara_ffn_desc* ffn, int32_t G, int32_t in_dtype,
                              epara_group_args* up_args, epara_group_args* down_args)
{
    if (G < 0) return EPARA_ERR_SHAPE;
    if (G == 0) return EPARA_OK;
    if (!ffn || !up_args || !down_args) return EPARA_ERR_NULL;
    if (in_dtype != EPARA_BF16 && in_dtype != EPARA_FP8_E4M3) return EPARA_ERR_DTYPE;
    const bool fp8 = in_dtype == EPARA_FP8_E4M3;
    for (int32_t g = 0; g < G; ++g) {
        const epara_ffn_desc& f = ffn[g];
        if (f.M < 0 || f.d_model <= 0 || f.d_ff <= 0) return EPARA_ERR_SHAPE;
        if (fp8 && !(f.s_x > 0.f && f.s_wgate > 0.f && f.s_wup > 0.f && f.s_h > 0.f && f.s_wdown > 0.f))
            return EPARA_ERR_SHAPE;
        epara_group_args u;
        std::memset(&u, 0, sizeof u);
        u.X = f.X; u.W = f.Wgate; u.W2 = f.Wup; u.bias = nullptr; u.Y = f.H;
        u.M = f.M; u.K = f.d_model; u.N = f.d_ff; u.act = EPARA_ACT_SWIGLU;
        u.scale = fp8 ? f.s_x * f.s_wgate : 1.f;
        u.scale2 = fp8 ? f.s_x * f.s_wup : 1.f;
        u.out_inv_scale = fp8 ? 1.f / f.s_h : 1.f;
        epara_group_args d;
        std::memset(&d, 0, sizeof d);
        d.X = f.H; d.W = f.Wdown; d.W2 = nullptr; d.bias = nullptr; d.Y = f.Y;
        d.M = f.M; d.K = f.d_ff; d.N = f.d_model; d.act = EPARA_ACT_NONE;
        d.scale = fp8 ? f.s_h * f.s_wdown : 1.f;
        d.scale2 = 1.f;
        d.out_inv_scale = 1.f;
        up_args[g] = u;
        down_args[g] = d;
    }
    return EPARA_OK;
}

}  // extern "C"
