/*
 * libepara -- grouped dense forward for co-located inference services on one MI355X.
 *
 *     Y_g = act_g( s_g * X_g W_g + b_g )          for g = 0 .. G-1, in ONE launch
 *
 * Vocabulary follows the paper (Sec. 3.1, "Task-Categorized Parallelism Allocator"):
 * a *service* is a deployed model, a *request* brings one or more rows (frames,
 * tokens), a *task* is a (request, service) pair.  Batching (BS) makes the rows of one
 * service's requests one ragged batch X_g [M_g, K_g]; multi-task (MT) lets several
 * services with different weights share the GPU -- here they share a kernel launch;
 * multi-frame (MF) only changes how many rows a request contributes.  The paper states
 * no layer arithmetic: the formula is the ordinary affine layer plus activation.
 * A *group* is one (service, layer) product.
 *
 * Conventions
 *   - plain C ABI; every entry point returns an epara_status (0 = EPARA_OK) unless noted;
 *     nothing aborts on bad input.
 *   - "h_" / "d_" prefixes say whether a pointer is host or device memory.
 *   - the caller owns every buffer and the stream; the library allocates no device memory
 *     and keeps no mutable global state (one exception, stated there: the scratch array of
 *     epara_grouped_chain_static).  Launch functions only enqueue work on `stream` (a
 *     hipStream_t passed as void*; NULL = default stream) and never synchronise; the one call
 *     that waits for the stream and copies to the host is epara_chain_status.
 *   - X_g and Y_g are dense row-major ([M,K] and [M,N]); device pointers must be 16-byte
 *     aligned and K*sizeof(element) must be a multiple of 16, and at most 8 MiB, for bf16/fp8
 *     inputs (ERR_ALIGN / ERR_SHAPE otherwise).
 *   - weights: logical W_g is [K,N] row-major.  fp32 kernels read that layout directly;
 *     bf16 / fp8 kernels read the tile-packed layout written by epara_pack_weights
 *     (done once when a service is placed on the GPU, ahead of its requests -- the paper
 *     pre-places models because loading costs far more than one task, Sec. 3.3).
 */
#ifndef EPARA_H
#define EPARA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    EPARA_OK = 0,
    EPARA_ERR_NULL = 1,      /* a required pointer is NULL */
    EPARA_ERR_SHAPE = 2,     /* negative/zero dimension, bad class table, tile outside its group, bad grid */
    EPARA_ERR_DTYPE = 3,     /* unsupported dtype / activation combination */
    EPARA_ERR_CAPACITY = 4,  /* an output array is too small (the needed size is still written) */
    EPARA_ERR_ALIGN = 5,     /* pointer or row pitch not 16-byte aligned */
    EPARA_ERR_HIP = 6        /* the HIP runtime refused the launch */
} epara_status;

typedef enum { EPARA_F32 = 0, EPARA_BF16 = 1, EPARA_FP8_E4M3 = 2 } epara_dtype;

/* EPARA_ACT_SWIGLU: the group has two weight matrices and computes
 * SiLU(s * X W) * (s2 * X W2); no bias. */
typedef enum {
    EPARA_ACT_NONE = 0, EPARA_ACT_RELU = 1, EPARA_ACT_GELU_ERF = 2,
    EPARA_ACT_GELU_TANH = 3, EPARA_ACT_SILU = 4, EPARA_ACT_SWIGLU = 5
} epara_act;

/* Sec. 3.1 "Task categories": latency- vs frequency-sensitive.  Metadata only: it never
 * changes a group's arithmetic. */
typedef enum { EPARA_CAT_LATENCY = 0, EPARA_CAT_FREQUENCY = 1 } epara_category;

typedef struct { int32_t M, K, N; int32_t act; int32_t has_bias; int32_t category; } epara_group_desc;

/* A group with M <= max_M (first such class wins) is cut into BM x BN output tiles.  split_K: 0, or the K
 * from which a single launch may visit a tile of this class in parts of K (see "Splitting K" below): a
 * weight-streaming tile in two, the panel tiles of a launch's last round in two to four. */
typedef struct { int32_t max_M; int32_t BM, BN; int32_t split_K; } epara_tile_class;

/* One output tile: rows [m0, m0+rows) x columns [n0, n0+cols) of group `group`. 24 bytes. */
typedef struct { int32_t group, m0, n0, rows, cols, cls; } epara_tile;

/* Per-group kernel arguments; the same bytes are used on the host (validation) and on the
 * device (the kernels read d_args[g]).  72 bytes. */
typedef struct {
    const void*  X;            /* device, [M,K] row-major, input dtype */
    const void*  W;            /* device, weights (layout: see above) */
    const void*  W2;           /* device, second weight matrix (EPARA_ACT_SWIGLU), else NULL */
    const float* bias;         /* device, fp32 [N], or NULL */
    void*        Y;            /* device, [M,N] row-major, output dtype */
    int32_t M, K, N;
    int32_t act;               /* epara_act */
    float scale;               /* s = s_x * s_w   (fp8 per-tensor scales; 1 otherwise) */
    float scale2;              /* s2 = s_x * s_w2 (EPARA_ACT_SWIGLU) */
    float out_inv_scale;       /* fp8 output: stored code = sat(RNE(y * out_inv_scale)); else 1 */
    int32_t reserved;          /* split_base[g] of epara_split_layout when the launch has split tiles, else ignored */
} epara_group_args;

/* Everything one launch needs.  h_* copies let the library validate shapes before it
 * enqueues anything; d_* copies are what the kernel reads. */
typedef struct {
    const epara_group_args* h_args;   /* host,   G entries */
    const epara_group_args* d_args;   /* device, G entries (same bytes) */
    const epara_tile*       h_tiles;  /* host,   n_tiles entries, canonical order */
    const epara_tile*       d_tiles;  /* device, same bytes */
    const int32_t*          d_order;  /* device, n_slots entries from epara_schedule_tiles */
    int64_t n_tiles;
    int64_t n_slots;
    int32_t n_workgroups;             /* the value the order was built for; becomes the grid size */
    int32_t G;
    void*   d_workspace;              /* device, 256-byte aligned, zeroed once (epara_workspace_init); NULL if nothing is split */
    int64_t workspace_bytes;          /* at least epara_split_workspace_bytes(n_split_tiles, n_panel_split_tiles) */
    int32_t n_split_tiles;            /* streaming tiles whose K is split over several visits (epara_split_layout) */
    int32_t n_panel_split_tiles;      /* panel tiles, the last ones of the tile table, likewise (epara_panel_split) */
} epara_launch;

/* ---- chains of launches in one kernel -----------------------------------------------------
 * The requests of a batch cross every layer of their service (Sec. 3.1: a batch is executed as a
 * whole), so consecutive grouped launches form a chain in which a group of one launch reads what a
 * group of the launch before wrote.  A chain runs as ONE persistent kernel: every workgroup walks
 * its list of the first launch ("phase"), then of the second, ...; a tile whose group reads a
 * produced tensor first waits until every tile of the producing group has been stored. */

/* What group g of a phase waits for: counter `counter` (or -1: nothing) must reach `need` = the
 * number of tiles of the producing group.  8 bytes; the same bytes on host and device. */
typedef struct { int32_t counter; int32_t need; } epara_chain_wait;

/* One phase of epara_schedule_chain: inputs as for epara_schedule_tiles, outputs order / n_slots. */
typedef struct {
    const epara_group_desc* groups;   /* host, G entries */
    const epara_tile_class* classes;  /* host, n_classes entries */
    const epara_tile*       tiles;    /* host, canonical table of (groups, classes) */
    int32_t*                order;    /* host, out: order_cap entries; NULL to query n_slots */
    int64_t n_tiles;
    int64_t order_cap;
    int64_t n_slots;                  /* out */
    int32_t G, n_classes, n_stream_classes, reserved;
} epara_phase_schedule;

/* One phase of epara_grouped_chain. */
typedef struct {
    const epara_launch*     launch;   /* host; all phases share n_workgroups */
    const epara_chain_wait* h_waits;  /* host, launch->G entries; NULL for a phase that waits for nothing */
    const epara_chain_wait* d_waits;  /* device, same bytes */
    int32_t out_dtype;
    int32_t counter_base;             /* tiles of group g of this phase count on counter counter_base + g */
} epara_chain_phase;

#define EPARA_MAX_CHAIN_PHASES 4

/* SwiGLU FFN of one service: Y = (SiLU(X Wgate) * (X Wup)) Wdown, H = the hidden
 * activations [M, d_ff] (caller-provided scratch, written then read). */
typedef struct {
    const void* X; const void* Wgate; const void* Wup; const void* Wdown;
    void* H; void* Y;
    int32_t M, d_model, d_ff;
    float s_x, s_wgate, s_wup, s_h, s_wdown;   /* per-tensor fp8 scales; ignored (1) otherwise */
} epara_ffn_desc;

/* One contiguous run of rows that moves between a request's own buffer and its place in the
 * ragged batch of its service (Sec. 3.1 BS / MF: a batch is formed from the rows of many requests
 * and its result rows go back to them).  40 bytes; the same bytes on host and device. */
typedef struct {
    const void* src;           /* device */
    void*       dst;           /* device */
    int64_t     bytes;         /* of the source; a multiple of 16, may be 0 */
    int64_t     first_chunk;   /* 16-KiB chunks of all earlier segments: sum ceil(bytes / 16384) */
    int32_t     group;         /* the service whose batch this run belongs to */
    int32_t     reserved;
} epara_segment;

/* ---- host side: batch accounting and planning (integers only, deterministic) ---------- */

/* Batch accounting (Sec. 3.1 BS / MF; Sec. 4.1): service g owns requests
 * request_off[g] .. request_off[g+1]-1, request r contributes request_rows[r] rows.
 * Writes M[g] = sum of its requests' rows and first_row[r] = rows of the same service
 * before request r.  ERR_SHAPE on a negative count, a decreasing offset or an M beyond int32. */
int32_t epara_batch_rows(const int32_t* request_rows, const int64_t* request_off, int32_t G,
                         int32_t* M, int64_t* first_row);

/* Batch forming (Sec. 3.1 BS / MF), the copy plan.  Requests are numbered as in epara_batch_rows;
 * request r of service g brings request_rows[r] rows of request_row_bytes[g] bytes in its own buffer
 * request_ptr[r]; the batch of service g is batch_ptr[g], dense rows of batch_row_bytes[g] bytes
 * (the same as request_row_bytes for a copy; a quarter or half of it when the rows are
 * quantised to one byte per element on the way).  With at = batch_ptr[g] + first_row[r] * batch_row_bytes[g]:
 *   to_batch != 0 (gather):  src = request_ptr[r], dst = at, bytes = request_rows[r] * request_row_bytes[g]
 *   to_batch == 0 (scatter): src = at, dst = request_ptr[r], bytes = request_rows[r] * batch_row_bytes[g]
 * first_chunk = running sum of ceil(bytes / 16384); group = g.  One segment per request, in request
 * order (requests without rows give bytes = 0).  *n_chunks receives the total.  Pointers are only
 * computed with, never dereferenced.
 * Errors: ERR_NULL; ERR_SHAPE for a negative count, a decreasing offset or a row size <= 0;
 * ERR_ALIGN if a row size is not a multiple of 16. */
int32_t epara_request_segments(const int32_t* request_rows, const int64_t* request_off, int32_t G,
                               const int64_t* request_row_bytes, const int64_t* batch_row_bytes,
                               const void* const* request_ptr, const void* const* batch_ptr, int32_t to_batch,
                               epara_segment* segments, int64_t* n_chunks);

/* Sec. 4.1, Eq. "DP group count" = ceil(required rate / rate of one group); -1 on bad input. */
int64_t epara_dp_group_count(int64_t rate_required, int64_t rate_of_one_group);
/* Sec. 4.1, Eq. "inter request count" = floor(BS / max inter-frame count); -1 on bad input. */
int64_t epara_inter_request_count(int64_t batch_size, int64_t max_inter_frame_count);

/* Allocation operators of Sec. 3.1 as bits. */
typedef enum { EPARA_OP_BS = 1, EPARA_OP_MT = 2, EPARA_OP_MP = 4, EPARA_OP_MF = 8, EPARA_OP_DP = 16 } epara_operator;

/* Sec. 3.1 "Performing operators to categories": the operators the allocator applies to a task of
 * `category` (epara_category) that fits one GPU (multi_gpu = 0) or needs several (multi_gpu != 0):
 *   latency,   one GPU : BS | MT            latency,   several : BS | MT | MP
 *   frequency, one GPU : MF | MT | BS       frequency, several : MF | MT | BS | DP | MP
 * -1 for an unknown category. */
int32_t epara_operator_set(int32_t category, int32_t multi_gpu);

/* Sec. 4.1 "DP and MF configuration": batching MF frames of a stream raises its latency from 1/fps to
 * MF/fps, so MF is set to the largest count the latency requirement allows:
 * floor(latency_us * fps_milli / 1e9), at least 1 (fps_milli = 1000 * frames per second).
 * -1 on a negative latency or a rate <= 0. */
int64_t epara_max_inter_frame_count(int64_t latency_us, int64_t fps_milli);

/* DP (Sec. 3.1): the frames of a task go to its DP groups in a round robin manner.  Frame j of the
 * n_frames frames that start at stream position first_frame goes to group (first_frame + j) mod n_groups.
 * Writes frames_per_group[n_groups] (may be NULL) and group_of_frame[n_frames] (may be NULL).
 * ERR_SHAPE for n_groups <= 0 or a negative count / position. */
int32_t epara_dp_deal(int64_t first_frame, int64_t n_frames, int64_t n_groups,
                      int64_t* frames_per_group, int32_t* group_of_frame);

/* ---- host side: request handling (Sec. 3.2) ------------------------------------------------- */

typedef enum {
    EPARA_HANDLE_TIMEOUT = 0,            /* the request already violates its SLO */
    EPARA_HANDLE_LOCAL = 1,              /* the locally placed services suffice */
    EPARA_HANDLE_OFFLOAD = 2,            /* sent on to *destination */
    EPARA_HANDLE_OFFLOAD_EXCEEDED = 3,   /* local resources insufficient and the offload count is used up */
    EPARA_HANDLE_INSUFFICIENT = 4        /* no server can take it, by this server's information */
} epara_handle_decision;

/* One scheduling decision of edge server `self` for one request, the steps of Sec. 3.2 in order:
 * timed out (now_us > deadline_us) -> TIMEOUT; local_can_serve != 0 -> LOCAL; otherwise
 * offload_count >= max_offload -> OFFLOAD_EXCEEDED; otherwise offload to a feasible server m != self
 * drawn with the probability of Eq. (1), idle[m] / sum of idle over the feasible servers, where
 * idle[m] = theoretical[m] - actual[m] (goodput the server could still add) must be positive and a
 * server is infeasible when the computation queued on it, queued_us[m], exceeds sync_delay_us +
 * slo_us; no feasible server -> INSUFFICIENT.  The draw is the caller's: u in [0, 1) picks the first
 * feasible m (ascending) whose cumulative share exceeds u.  Writes *decision (and *destination, -1
 * unless OFFLOAD).  ERR_NULL / ERR_SHAPE (n_servers <= 0, self outside, u outside [0, 1)). */
int32_t epara_handle_request(int64_t now_us, int64_t deadline_us, int32_t local_can_serve,
                             int32_t offload_count, int32_t max_offload,
                             const double* theoretical, const double* actual, const int64_t* queued_us,
                             int32_t n_servers, int32_t self, int64_t sync_delay_us, int64_t slo_us, double u,
                             int32_t* decision, int32_t* destination);

/* ---- host side: service placement (Sec. 3.3, Alg. 1 and 2) --------------------------------- */

/* The objective phi(Theta) of Eq. "optimal": how many requests of the period the placement list
 * Theta (placements[0..n), opaque non-negative ids of "service l on server n") lets the request
 * handler satisfy.  Supplied by the caller (it owns the request list and the handling model);
 * must be deterministic.  `user` is passed through. */
typedef double (*epara_phi_fn)(const int32_t* placements, int32_t n, void* user);

/* Alg. 2, submodular placement for full models: starting from theta0, repeatedly evaluate
 * phi(Theta + delta) for every candidate delta -- all of `candidates` each round if is_set != 0 (a
 * placement may be chosen again: replicas), else those not chosen yet (a list, without
 * replacement) -- and append one that maximises it (ties: the earliest candidate; the paper says
 * "arbitrary").  The round's addition is kept while phi does not decrease (keep_equal != 0, step S1
 * of Alg. 1) or while it strictly increases (keep_equal == 0); the first addition that fails the
 * test is dropped and the list before it is returned, as is the list when no candidate is left.
 * Writes theta_out[0..*n_out) (theta0 first).  Errors: ERR_NULL; ERR_SHAPE for negative counts or
 * ids; ERR_CAPACITY when the list would outgrow cap (also bounds a phi that never stops improving). */
int32_t epara_place_full_models(const int32_t* candidates, int32_t n_candidates, int32_t is_set, int32_t keep_equal,
                                const int32_t* theta0, int32_t n0, epara_phi_fn phi, void* user,
                                int32_t* theta_out, int32_t cap, int32_t* n_out);

/* Alg. 1, state-aware service placement: S1 places the prioritised partial configurations (a list,
 * kept while phi does not decrease), S2 places from the set X of all (service, server)
 * placements, S3 from the set X_dot of placements on the hypothetical server that aggregates every
 * GPU (multi-GPU parallelism across servers); each step continues from the previous list. */
int32_t epara_place_services(const int32_t* partial, int32_t n_partial, const int32_t* X, int32_t n_x,
                             const int32_t* X_dot, int32_t n_xdot, epara_phi_fn phi, void* user,
                             int32_t* theta_out, int32_t cap, int32_t* n_out);

/* ---- host side: the placement objective by event-driven simulation (Sec. 3.3, Sec. 5) -------- */

/* One user request of the period.  32 bytes. */
typedef struct {
    int64_t arrival_us;        /* when the user sends it to server `origin` */
    int64_t slo_us;            /* latency SLO: it must be finished by arrival_us + slo_us */
    int32_t service;           /* l */
    int32_t origin;            /* n */
    int32_t frames;            /* >= 1: it occupies an instance for frames * c_ln microseconds */
    int32_t fps_milli;         /* 0: latency-sensitive; > 0: frequency-sensitive, 1000 * the frame rate its SLO asks for */
} epara_sim_request;

typedef struct {
    const int64_t* compute_us; /* c_ln, [n_services * n_servers] row-major (service major): the time one frame of
                                  service l takes on server n, from a lookup table (measured); <= 0: cannot run there */
    int64_t hop_us;            /* transmission time of one offload hop */
    int64_t sync_delay_us;     /* t: period and delay of the state synchronisation, > 0 */
    int32_t n_servers, n_services;
    int32_t max_offload;       /* offload count at which the handler gives up */
    int32_t reserved;
} epara_sim_config;

typedef struct {
    double  satisfied;         /* phi(Theta): requests served within their SLO; frames of frequency-sensitive requests
                                  count in proportion to the achieved rate (Sec. 3.3) */
    int64_t local, offloaded, timeout, offload_exceeded, insufficient;   /* handler decisions taken */
} epara_sim_result;

/* The lookup table c_ln of Sec. 3.3 / Sec. 5 from measured passes: service l was measured on the
 * reference GPU at ms_per_pass[l] milliseconds for a pass that serves requests_per_pass[l] requests
 * (what bench.py reports per mix), and server n runs at server_speed[n] times the reference GPU's
 * speed (1 = the same GPU; <= 0: it cannot run services).  compute_us[l * n_servers + n] =
 * ceil(1000 * ms_per_pass[l] / requests_per_pass[l] / server_speed[n]), at least 1; 0 where the server
 * cannot run it.  ERR_NULL; ERR_SHAPE for counts < 0, a time <= 0 or a request count <= 0. */
int32_t epara_compute_table(const double* ms_per_pass, const int32_t* requests_per_pass, int32_t n_services,
                            const double* server_speed, int32_t n_servers, int64_t* compute_us);

/* phi(Theta) of Eq. "optimal" for the placement list placements[0..n) (id = l * n_servers + n, one
 * service instance per entry, repeats = replicas), by replaying the period's requests through the
 * handler of Sec. 3.2 (epara_handle_request) event by event; nothing is executed, computation times
 * come from the table (Sec. 3.3: c_ln; Sec. 5: lookup tables indexed by GPU and service).  Model:
 *   - an instance serves one request at a time in the order they were bound to it;
 *   - "locally sufficient" = the instance of (l, n) that is free first finishes the request by its
 *     deadline; the request is bound to it at once and counts as one satisfied request;
 *   - a frequency-sensitive request (fps_milli > 0) is a stream of `frames` frames, each counting as a
 *     request (Sec. 3.3: 120 frames wanted at 60 fps, served at 30 fps, count 120 * 30 / 60 = 60): it is
 *     locally sufficient wherever an instance of (l, n) exists, is bound to the one that is free first, and
 *     adds frames * min(1, achieved / required) with achieved = frames * 1e6 / (finish - arrival_us) per second;
 *   - every sync_delay_us = t, at time j*t, each server publishes per service its completions in
 *     ((j-1)t, jt] and when its first instance is free; at time `now` the others know snapshot
 *     J = floor(now / t) - 1 (J < 1: nothing yet, zeros): theoretical goodput = instances * 1e6 / c_lm,
 *     actual = completions of that window * 1e6 / t, queued = max(0, first free time - J*t);
 *   - servers a request has visited are never destinations (no loops); a hop takes hop_us;
 *   - the k-th offloading decision of request r uses draws[r * max_offload + k] in [0, 1).
 * Events are handled in (time, sequence) order; sequence = request index for arrivals from users,
 * then in order of creation for offloaded arrivals.  Requests need not be sorted.
 * Errors: ERR_NULL; ERR_SHAPE for counts <= 0 (servers, services, t), negative counts, ids, frames < 1
 * a negative fps_milli or a draw outside [0, 1). */
int32_t epara_simulate(const epara_sim_config* config, const int32_t* placements, int32_t n_placements,
                       const epara_sim_request* requests, int64_t n_requests, const double* draws,
                       epara_sim_result* result);

/* Group planning (Sec. 3.1: the allocator decides the parallel mode of each task; BS / MF fix the
 * rows of a service's batch, MT puts the services on one GPU): the single-GPU part of that decision.
 *   row_off[g] = sum_{h<g} M_h ; x_off[g] = sum_{h<g} M_h K_h ; y_off[g] = sum_{h<g} M_h N_h
 *   (each G+1 entries; x_off / y_off are element offsets for callers that pack groups
 *   back to back), tile class of g = first class with M_g <= max_M, and the canonical tile
 *   table: g ascending, then m0, then n0, rows = min(BM, M_g - m0), cols = min(BN, N_g - n0).
 * M_g = 0 and G = 0 are legal (no tiles).  tiles may be NULL to query *n_tiles only.
 * Errors: NULL groups (G > 0) / classes / n_tiles -> ERR_NULL; M < 0, K <= 0, N <= 0, G < 0,
 * BM or BN <= 0, max_M not strictly increasing, or a group no class admits -> ERR_SHAPE;
 * tiles_cap < needed -> ERR_CAPACITY with *n_tiles written. row_off/x_off/y_off may be NULL. */
int32_t epara_plan_groups(const epara_group_desc* groups, int32_t G,
                          const epara_tile_class* classes, int32_t n_classes,
                          int64_t* row_off, int64_t* x_off, int64_t* y_off,
                          epara_tile* tiles, int64_t tiles_cap, int64_t* n_tiles);

/* The scheduler's cost model, in one place.  A streaming tile costs
 *     K * (EPARA_COST_PER_COLUMN * cols * (2 for EPARA_ACT_SWIGLU groups) + EPARA_COST_PER_ROW * BM for classes with BM >= 32)
 * (weight columns streamed from HBM; activation rows re-read from L2 through the LDS: workgroups of the
 * decode mix that stream the same 1.41 MB of weights take 62 / 72 / 83 us with tiles of the 16- / 32- /
 * 64-row class, i.e. a row of the larger classes costs a third of a weight column and the rows of the
 * 16-row class disappear under the weight stream); a panel tile costs EPARA_COST_PANEL * K. */
#define EPARA_COST_PER_COLUMN 6
#define EPARA_COST_PER_ROW 2
#define EPARA_COST_PANEL 2040
#define EPARA_COST_PARTIAL 24

/* Splitting K.  A streaming tile of a class with BM >= 32 streams its weights while re-reading BM activation
 * rows per weight column, which is cheapest with wide tiles; wide tiles of a long K are too coarse to balance,
 * so the scheduler can cut their K instead: a tile of a streaming class with split_K > 0 and K >= split_K is
 * visited P = EPARA_SPLIT_PARTS times, each visit multiplying one contiguous part of K (part j of P covers the
 * steps floor(S j / P) .. floor(S (j+1) / P) - 1 of the S = ceil(K / step) steps of 128 bytes of K).  The visits
 * leave their sums in a device workspace; a workgroup counts its visits at the tiles' counters when its list
 * ends, and whoever counts last at a tile adds the parts in index order (a fixed order: the result does not
 * depend on timing or on the grid) and runs the epilogue.  An entry of the visit order then is
 * tile | part << 24 | (P - 1) << 28  (P = 1: just the tile; the format leaves room for up to
 * EPARA_SPLIT_MAX_PARTS).  Only single launches are split (epara_schedule_tiles); the phases of a chain are not.
 * Every visit costs a few microseconds of its own (another start of the weight stream, the sums' trip through
 * memory).  Measured on the decode mix: two parts pay for bf16 from K = 8192 on (EPARA_SPLIT_K_BF16, what
 * epara_kernel_classes puts into the 32- and 64-row classes); four parts, a shorter K, or fp8 (half the bytes
 * per visit) do not, so the fp8 tables carry split_K = 0. */
#define EPARA_SPLIT_PARTS 2
#define EPARA_SPLIT_K_BF16 8192
#define EPARA_SPLIT_MAX_PARTS 4
#define EPARA_SPLIT_STRIDE 32768      /* bytes of partial sums per (split streaming tile, part) */

/* Panel tiles can be split the same way, for another reason: a launch of n equal panel tiles on W workgroups
 * ends with a round of m = n mod W tiles that leaves W - m workgroups idle for a whole tile.  When the launch
 * holds nothing but panel tiles of one class with split_K > 0 and one K >= split_K, of groups without
 * EPARA_ACT_SWIGLU (a down projection; epara_kernel_classes sets EPARA_PANEL_SPLIT_K for the plain bf16
 * panel class, 0 for the gated one, for fp8, whose visits are half as long, and for fp32), those m tiles -- the
 * last m of the canonical table -- are visited in parts of K instead: tile i of them in P_i parts, part j of P
 * covering the units floor(U j / P) .. floor(U (j+1) / P) - 1 of the U = ceil(ceil(K / stage) / 4) units of four
 * 64-byte stages.  The P_i are chosen among
 *   (a) every tile in P parts, P = 2 .. EPARA_SPLIT_MAX_PARTS: time ceil(m P / W) * (cost / P + EPARA_COST_PANEL_PARTIAL);
 *   (b) k = 1 .. EPARA_SPLIT_MAX_PARTS parts per workgroup, Q = k W parts in all with 2 m <= Q <= m EPARA_SPLIT_MAX_PARTS
 *       and Q not a multiple of m: the first m - Q mod m tiles in P = floor(Q / m) parts, the others in P + 1; time =
 *       the most loaded of W level workgroups when the Q parts, the larger ones first, each go to the least loaded;
 * by the smallest time, in this order on ties, and only below 0.9 * cost (cost = EPARA_COST_PANEL * K).
 * A visit leaves its 256 x 256 fp32 sums (EPARA_PANEL_SPLIT_STRIDE bytes) in the workspace, behind the streaming
 * tiles' slots; counting and the addition in index order work as for streaming tiles.  epara_panel_split states
 * the decision (*parts = P of the first tiles, *n_more = how many of the last tiles get P + 1); it depends on the
 * grid size. */
#define EPARA_PANEL_SPLIT_STRIDE 262144   /* bytes of partial sums per (split panel tile, part) */
#define EPARA_PANEL_SPLIT_K 1024          /* every part then holds whole units of four stages, bf16 or fp8 */
#define EPARA_COST_PANEL_PARTIAL 1020000  /* a part's trip through memory, in cost units (about 500 elements of K) */
int32_t epara_panel_split(const epara_group_desc* groups, int32_t G,
                          const epara_tile_class* classes, int32_t n_classes, int32_t n_stream_classes,
                          int32_t n_workgroups, int32_t* n_panel_split_tiles, int32_t* parts, int32_t* n_more);

/* Bytes of the workspace of a launch with n_split_tiles split streaming tiles and n_panel_split_tiles split
 * panel tiles: 4 bytes of counter per split tile, rounded up to 256, then EPARA_SPLIT_MAX_PARTS parts of
 * EPARA_SPLIT_STRIDE bytes per streaming tile, then EPARA_SPLIT_MAX_PARTS parts of EPARA_PANEL_SPLIT_STRIDE bytes
 * per panel tile; 0 if both counts are 0, -1 if one is negative. */
int64_t epara_split_workspace_bytes(int32_t n_split_tiles, int32_t n_panel_split_tiles);
#define EPARA_ORDER_ENTRY(tile, part, parts) ((int32_t)((tile) | ((part) << 24) | (((parts) - 1) << 28)))
#define EPARA_ORDER_TILE(entry) ((entry) & 0xFFFFFF)

/* Where the split tiles of a launch meet: split_base[g] (G entries) = index of the first split tile of
 * group g among all split tiles of the launch (its tiles follow in n0 order), or -1 if the tiles of g are
 * not split; *n_split_tiles = their number; *workspace_bytes = epara_split_workspace_bytes(n_split_tiles, 0).
 * The caller writes split_base[g] into epara_group_args.reserved, sets epara_launch.n_split_tiles (and
 * n_panel_split_tiles from epara_panel_split) and provides a workspace of
 * epara_split_workspace_bytes(n_split_tiles, n_panel_split_tiles) bytes, zeroed once with epara_workspace_init
 * (a launch leaves its counters zero).  epara_plan_launch does all of this.
 * More than 2^24 tiles -> ERR_SHAPE. */
int32_t epara_split_layout(const epara_group_desc* groups, int32_t G,
                           const epara_tile_class* classes, int32_t n_classes, int32_t n_stream_classes,
                           int32_t* split_base, int32_t* n_split_tiles, int64_t* workspace_bytes);

/* Zeroes a launch workspace (one small kernel on `stream`). */
int32_t epara_workspace_init(void* d_workspace, int64_t bytes, void* stream);

/* Visit order of the persistent workgroups.  Workgroup b of W = n_workgroups visits slots
 * b, b + W, b + 2W, ...; order[slot] is a tile index (with the part of K in its upper bits when the tile
 * is split) or -1 (idle).  Every workgroup gets a list
 * of tiles; slot j*W + b holds the j-th entry of workgroup b's list; *n_slots = W * (longest list).
 * The first n_stream_classes classes of the table are weight-streaming classes (small batches,
 * bandwidth bound), the others are panel classes (matrix-core bound).
 *   1. panel tiles: classes by descending BM*BN (ties: lower class), inside a class groups by
 *      descending K (ties: lower group), inside a group panels of panel_m x panel_n tiles,
 *      n-panel outermost, m fastest inside a panel.  Each tile of that sequence goes to the workgroup
 *      with the smallest accumulated cost (EPARA_COST_PANEL * K per panel tile); among equally loaded
 *      workgroups the smallest die-major rank wins, rank r standing for workgroup (r mod (W/X)) * X +
 *      r div (W/X)  (X = n_xcd).  Tiles of equal cost therefore go round robin, the l-th to rank l mod W,
 *      so that the W/X workgroups of one compute die (workgroup b runs on die b mod X) work on
 *      neighbouring tiles and share operands in that die's L2; where K differs between the groups of a
 *      launch, a workgroup that got a long tile gets fewer of the short ones.
 *   2. streaming tiles, longest first: costs as defined above (EPARA_COST_*); a tile that is split (see
 *      "Splitting K") gives P items, each of cost / P + EPARA_COST_PARTIAL * BM * cols (* 2 for
 *      EPARA_ACT_SWIGLU groups; the partial sums it writes and the last visit reads); items by descending
 *      cost (ties: lower tile index, then lower part) each go to the
 *      workgroup with the smallest accumulated cost (ties: lower workgroup), after that
 *      workgroup's panel tiles.
 * order may be NULL to query *n_slots.  W must be a positive multiple of X;
 * 0 <= n_stream_classes <= n_classes.  Errors as for epara_plan_groups; a tile table that is not
 * the canonical one of (groups, classes) gives ERR_SHAPE. */
int32_t epara_schedule_tiles(const epara_group_desc* groups, int32_t G,
                             const epara_tile_class* classes, int32_t n_classes, int32_t n_stream_classes,
                             const epara_tile* tiles, int64_t n_tiles,
                             int32_t n_workgroups, int32_t n_xcd, int32_t panel_m, int32_t panel_n,
                             int32_t* order, int64_t order_cap, int64_t* n_slots);

/* Visit orders for a chain of launches that one kernel runs phase after phase (a workgroup's
 * list of phase p+1 follows its list of phase p).  The rule of epara_schedule_tiles with the
 * workgroup loads shared by all phases, so that a workgroup with much work in one phase gets less in
 * another:
 *   1. panel tiles phase by phase, each phase's sequence as in epara_schedule_tiles, on the loads
 *      accumulated over the phases before.
 *   2. the streaming tiles of ALL phases together, by descending cost (ties: earlier phase, then
 *      lower tile index), each onto the workgroup with the smallest accumulated cost (ties: lower
 *      workgroup); it joins that workgroup's list of its own phase, after the panel tiles.
 * Per phase: n_slots = W * (longest list of that phase) and order as in epara_schedule_tiles.
 * With n_phases = 1 this IS epara_schedule_tiles.  Errors as there; ERR_CAPACITY (every n_slots
 * written) if an order array is too small. */
int32_t epara_schedule_chain(epara_phase_schedule* phases, int32_t n_phases,
                             int32_t n_workgroups, int32_t n_xcd, int32_t panel_m, int32_t panel_n);

/* What epara_plan_launch decided and how large its outputs are. */
typedef struct {
    epara_tile_class classes[4];      /* the class table the launch was cut with */
    int32_t n_classes, n_stream_classes;
    int32_t narrow;                   /* 1: the narrow table (see epara_kernel_classes) */
    int32_t gated;                    /* 1: every group is EPARA_ACT_SWIGLU */
    int64_t n_tiles, n_slots;
    int64_t makespan;                 /* cost of the most loaded workgroup under the cost model */
    int64_t workspace_bytes;          /* epara_split_workspace_bytes of the two counts below */
    int32_t n_split_tiles, n_panel_split_tiles;
} epara_launch_plan;

/* The whole planning decision of one launch (Sec. 3.1: the parallel mode of each task): picks the class
 * table -- the wide one, or the narrow one when some batch has more than 32 rows and the narrow
 * table's schedule has the smaller makespan under the cost model (ties: wide) -- then plans
 * (epara_plan_groups) and schedules (epara_schedule_tiles) with it.  The groups must be all
 * EPARA_ACT_SWIGLU or none (ERR_DTYPE).  *plan is always written (sizes included); tiles / order are
 * written when given and large enough, else ERR_CAPACITY (give NULL and 0 to ask for the sizes only;
 * that returns EPARA_OK).  row_off / x_off / y_off and split_base (G entries, epara_split_layout) may be NULL.
 * plan->n_split_tiles, n_panel_split_tiles and workspace_bytes say what the launch needs for tiles visited in
 * parts of K ("Splitting K").
 * Other errors as for the two calls. */
int32_t epara_plan_launch(const epara_group_desc* groups, int32_t G, int32_t in_dtype,
                          int32_t n_workgroups, int32_t n_xcd, int32_t panel_m, int32_t panel_n,
                          int64_t* row_off, int64_t* x_off, int64_t* y_off,
                          epara_tile* tiles, int64_t tiles_cap, int32_t* order, int64_t order_cap,
                          int32_t* split_base, epara_launch_plan* plan);

/* One phase of epara_plan_chain: in: groups, G, producer (per group the group of the phase before whose
 * output it reads, or -1; NULL: the phase waits for nothing); out: tiles, order, waits (G entries; may
 * be NULL when producer is), counter_base, plan. */
typedef struct {
    const epara_group_desc* groups;
    const int32_t*          producer;
    epara_tile*             tiles;
    int32_t*                order;
    epara_chain_wait*       waits;
    int64_t tiles_cap, order_cap;
    int32_t G;
    int32_t counter_base;             /* out: the sum of G over the phases before */
    epara_launch_plan plan;           /* out */
} epara_chain_plan_phase;

/* The planning decision of a chain (epara_grouped_chain): for every phase the wide or the narrow table
 * (phases with a batch of more than 32 rows have the choice), taken jointly: every combination is
 * scheduled with epara_schedule_chain and replayed under the cost model -- a workgroup walks its
 * lists phase after phase, a tile starts when its workgroup is free and, if its group waits, when the
 * last tile of the producing group has ended -- and the combination whose last workgroup finishes first
 * is kept (ties: the earlier combination, wide before narrow, first phase varying slowest).  Then tiles,
 * orders, waits (epara_chain_waits) and counter bases are written as for epara_plan_launch; all sizes
 * are always written, ERR_CAPACITY if an array that was given is too small. */
int32_t epara_plan_chain(epara_chain_plan_phase* phases, int32_t n_phases, int32_t in_dtype,
                         int32_t n_workgroups, int32_t n_xcd, int32_t panel_m, int32_t panel_n, int64_t* finish);

/* The waits of one phase of a chain: producer[g] = the group of the phase before whose output Y is
 * group g's input X, or -1.  waits[g] = { counter_base + producer[g], number of tiles of that group
 * in producer_tiles } or { -1, 0 }; counter_base is the producing phase's.  Host only.
 * ERR_SHAPE for an index outside [-1, G_producer) or a tile whose group is outside. */
int32_t epara_chain_waits(const epara_tile* producer_tiles, int64_t n_producer_tiles, int32_t G_producer,
                          int32_t counter_base, const int32_t* producer, int32_t G_consumer,
                          epara_chain_wait* waits);

/* The tile classes the kernels implement for an input dtype (gated = EPARA_ACT_SWIGLU
 * launches, whose BN counts hidden columns).  Writes up to cap classes, *n_classes = count and
 * *n_stream_classes = how many of them (the first ones) are weight-streaming classes.
 * bf16 / fp8 have two tables: the wide one (narrow = 0) gives batches of 33..64 rows tiles of 128
 * (gated: 64) columns, which halves the activation re-reads; the narrow one (narrow = 1) gives
 * them 64 (gated: 32) columns, for launches with too few columns to keep every workgroup busy
 * with wide tiles.  A launch may use either.  fp32: batches of up to 16 rows in 16 x 64 tiles (the sum
 * over K is formed in four contiguous quarters that are added in order), larger ones in 64 x 64
 * tiles (K ascending). */
int32_t epara_kernel_classes(int32_t in_dtype, int32_t gated, int32_t narrow,
                             epara_tile_class* classes, int32_t cap, int32_t* n_classes,
                             int32_t* n_stream_classes);

/* Fills the two phases' group arguments of a SwiGLU FFN from per-service descriptors:
 * up_args[g]   : X -> H, W = Wgate, W2 = Wup, act = SWIGLU, K = d_model, N = d_ff
 * down_args[g] : H -> Y, W = Wdown, act = NONE, K = d_ff, N = d_model
 * with the fp8 scale products filled in (all 1 for other dtypes).  Host only. */
int32_t epara_ffn_swiglu_args(const epara_ffn_desc* ffn, int32_t G, int32_t in_dtype,
                              epara_group_args* up_args, epara_group_args* down_args);

/* ---- device side -------------------------------------------------------------------- */

/* An upper bound of the device workspace a launch of these groups on n_workgroups workgroups needs, whichever
 * class table the plan picks (epara_plan_launch reports the exact size): the larger of the two tables' needs;
 * 0 when no tile would be split (fp32 launches, batches of at most 16 rows, short K, full last rounds).  -1 for
 * a bad dtype, G < 0, n_workgroups <= 0 or a mixture of EPARA_ACT_SWIGLU and other groups. */
int64_t epara_workspace_bytes(const epara_group_desc* groups, int32_t G, int32_t in_dtype, int32_t n_workgroups);

/* Bytes of the packed form of a [K,N] weight matrix (fp32: K*N*4, unchanged layout). */
int64_t epara_packed_weight_bytes(int32_t K, int32_t N, int32_t dtype);

/* Packs d_W ([K,N] row-major, `dtype`) into d_packed for the bf16 / fp8 kernels:
 * 1 KiB fragments of 16 columns x (64 bytes of K), fragment (nb, ks) at
 * ((nb * KSP + ks) * 1024) bytes, KSP = ceil(K/KF) rounded up to a multiple of 4, KF = 32 (bf16)
 * or 64 (fp8); inside a fragment the 16-byte chunk (q*16 + r) holds
 * W[ks*KF + q*KF/4 ... +KF/4-1][nb*16 + r]; zero padded, the padding stages included.
 * fp32: plain copy.  Enqueues one kernel. */
int32_t epara_pack_weights(const void* d_W, int32_t K, int32_t N, int32_t dtype,
                           void* d_packed, int64_t packed_bytes, void* stream);

/* The MT operator of Sec. 3.1 on one GPU (several services with their own weights share it; here
 * they share a launch), over batches formed by BS / MF; the weights are already resident (Sec. 3.3
 * pre-placement, epara_pack_weights).
 * Y_g = act_g(s_g X_g W_g + b_g) for all groups of the launch, in one persistent kernel
 * that walks the device tile table in the scheduled order; bias, activation, SwiGLU gating
 * and the output cast are fused in the epilogue.  Accumulation is fp32 in a fixed order
 * (bit-reproducible, independent of n_workgroups).
 * in_dtype / out_dtype: F32 -> F32; BF16 -> BF16; FP8_E4M3 -> BF16 or FP8_E4M3.
 * n_tiles = 0 enqueues nothing.  Validates h_args / h_tiles first: ERR_NULL, ERR_SHAPE,
 * ERR_DTYPE, ERR_ALIGN as described at the top; ERR_HIP if the launch fails. */
int32_t epara_grouped_forward(const epara_launch* launch, int32_t in_dtype, int32_t out_dtype,
                              void* stream);

/* Two dependent grouped launches of the same batches (Sec. 3.1: a batch crosses its service's layers
 * as a whole; MT across the services):
 * Y_g = (SiLU(X_g Wgate_g) * (X_g Wup_g)) Wdown_g for all services: phase `up` (gated
 * launch writing H in h_dtype) then phase `down` (reading H), enqueued back to back on
 * `stream`.  in_dtype BF16: h_dtype = out_dtype = BF16.  in_dtype FP8_E4M3: h_dtype =
 * FP8_E4M3 (codes sat(RNE(h / s_h))), out_dtype = BF16. */
int32_t epara_grouped_ffn_swiglu(const epara_launch* up, const epara_launch* down,
                                 int32_t in_dtype, int32_t h_dtype, int32_t out_dtype, void* stream);

/* Bytes of the device workspace of a chain with n_counters completion counters (the sum of G
 * over its phases): a 16-byte header (error flag, exit count) and the counters. */
int64_t epara_chain_workspace_bytes(int32_t n_counters);

/* Zeroes a chain workspace (one small kernel).  Needed once: a chain kernel leaves the counters
 * zero again when its last workgroup exits. */
int32_t epara_chain_workspace_init(void* d_workspace, int64_t bytes, void* stream);

/* The n_phases (1..EPARA_MAX_CHAIN_PHASES) launches of a chain in ONE persistent kernel of
 * n_workgroups workgroups: the same tiles, arithmetic and results as epara_grouped_forward called
 * phase by phase (bit-identical, except that the phases of a chain are never visited in parts of K, see
 * "Splitting K"), without the launch boundaries: a workgroup that finishes its
 * share of a phase goes on with the next phase at once, and a tile of group g waits only for the
 * group that produces its input (phase[p].h_waits[g]).  Completion is counted per group in
 * d_workspace (counter counter_base + g of phase p rises by the tiles a workgroup has stored, after
 * its stores, which go through to memory, have completed; a workgroup may hold back the counts of up
 * to two groups until it starts a third or ends the phase); counter ranges of different phases
 * must not overlap.  The kernels exist for chains without EPARA_ACT_SWIGLU groups (up to
 * EPARA_MAX_CHAIN_PHASES phases) and for the two phases of a SwiGLU FFN (gate/up, then down);
 * other mixtures of gated and plain phases -> ERR_DTYPE.  Every phase but the last must store
 * in_dtype (the next phase reads it) -> ERR_DTYPE.
 * Requirements beyond epara_grouped_forward's, checked before anything is enqueued: every phase has
 * the same n_workgroups, which must not exceed what the GPU keeps resident at once (a waiting
 * workgroup must never keep the one it waits for from running) -> ERR_SHAPE; a wait must name a
 * counter of the phase before, with need = that group's tile count, and the waiting group's X must
 * be that group's Y with matching shape -> ERR_SHAPE; a tensor that is waited for must own its cache
 * lines (consumers invalidate nothing after a wait, so a line it shared with another tensor of the
 * chain could be cached before it was written): it must start on a 128-byte boundary, and no other
 * tensor of the chain (X, Y, weights, bias of any group) may overlap the rest of its last 128-byte
 * line -> ERR_ALIGN; workspace too small -> ERR_CAPACITY.
 * A wait polls at most spin_limit times (0 = the default, some seconds); if it runs out the kernel
 * sets the error flag, goes on without the data and still terminates, and the outputs of the chain
 * are invalid: read the flag with epara_chain_status.  Two chains that use one workspace must not
 * overlap in time.
 * Meant for passes of long (panel-class) tiles submitted once; for passes of short weight-streaming tiles
 * (decode-sized batches, small models) separate launches are faster on this GPU, because every dependency
 * costs a poll, a drained pipeline and a fresh start of the weight stream, more than the launch boundary
 * it removes. */
int32_t epara_grouped_chain(const epara_chain_phase* phases, int32_t n_phases, int32_t in_dtype,
                            void* d_workspace, int64_t workspace_bytes, uint32_t spin_limit, void* stream);

/* epara_grouped_chain for callers that cannot allocate device memory or bring a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same chain, the
 * same kernels and results, with the completion counters in a device array that is part of the
 * library (EPARA_STATIC_CHAIN_COUNTERS counters, 16 KiB; every GPU the library runs on holds its copy
 * until the process ends).  Enqueues, on `stream`: a small kernel that zeroes the header and the
 * counters the chain uses (the array keeps what the last call left), the chain kernel, and, if d_flag
 * is given, a kernel that copies the error flag (0 = every wait ended normally) to *d_flag (device
 * memory of the caller, 4-byte aligned).  Calls no allocation routine and never synchronises.
 * Errors as for epara_grouped_chain; a chain with more than EPARA_STATIC_CHAIN_COUNTERS counters
 * (the sum of G over its phases) -> ERR_CAPACITY.  Every call on a GPU shares that GPU's array: two
 * calls that overlap in time on one GPU (different streams) race and their results are undefined. */
#define EPARA_STATIC_CHAIN_COUNTERS 4092
int32_t epara_grouped_chain_static(const epara_chain_phase* phases, int32_t n_phases, int32_t in_dtype,
                                   uint32_t spin_limit, int32_t* d_flag, void* stream);

/* Waits for `stream`, then *flag = the workspace's error flag (0 = every wait of every chain since
 * the last call ended normally) and clears it. */
int32_t epara_chain_status(void* d_workspace, void* stream, int32_t* flag);

/* ---- device side: the step before and after the path (batch forming) --------------------- */

/* Copies every segment (gather of request rows into the batches, or scatter of result rows back):
 * dst[0..bytes) = src[0..bytes).  One kernel; a workgroup copies 16-KiB chunks and finds the
 * segment of a chunk by bisection over first_chunk.  n_segments = 0 or n_chunks = 0 enqueues nothing.
 * Validates h_segments: ERR_NULL (src or dst NULL with bytes > 0), ERR_SHAPE (negative bytes,
 * first_chunk not the running sum, n_chunks not the total), ERR_ALIGN (pointer or bytes not a
 * multiple of 16). */
int32_t epara_copy_segments(const epara_segment* h_segments, const epara_segment* d_segments,
                            int64_t n_segments, int64_t n_chunks, void* stream);

/* Gather with dynamic per-tensor fp8 quantisation: the rows of all requests of service g are one
 * tensor; d_amax[g] = max |x| over it, d_scale[g] = d_amax[g] / 448 (1 if the tensor is all zero or
 * empty), and dst receives the E4M3 codes sat(RNE(x * (1 / d_scale[g]))) (reciprocal, product and
 * rounding in fp32, the same form as the forward path's out_inv_scale; one byte per source
 * element, so dst holds bytes / sizeof(src element)).  src_dtype is
 * EPARA_F32 or EPARA_BF16.  d_amax and d_scale are float[G] outputs in device memory.  Three
 * kernels on `stream`: clear, amax (integer max on the bit patterns: order independent),
 * quantise (which also writes the scales).  Validation as for epara_copy_segments plus ERR_DTYPE and ERR_SHAPE for a
 * group index outside [0, G).  A NaN in the input gives unspecified codes for its tensor. */
int32_t epara_quantize_segments_e4m3(const epara_segment* h_segments, const epara_segment* d_segments,
                                     int64_t n_segments, int64_t n_chunks, int32_t G, int32_t src_dtype,
                                     float* d_amax, float* d_scale, void* stream);

/* Writes scale products computed on the device into the device copy of the group arguments, so
 * that a launch can use scales that only exist in device memory (dynamic quantisation):
 *   d_args[g].scale = d_sx[g] * d_sw[g];  if d_sw2: d_args[g].scale2 = d_sx[g] * d_sw2[g];
 *   if d_sout: d_args[g].out_inv_scale = 1 / d_sout[g].
 * d_sx, d_sw: float[G] (required); d_sw2, d_sout may be NULL (fields left as they are).  The host
 * copy h_args is not touched: launch validation does not read the scale fields. */
int32_t epara_patch_scales(epara_group_args* d_args, int32_t G, const float* d_sx, const float* d_sw,
                           const float* d_sw2, const float* d_sout, void* stream);

/* ---- device side: between the dense layers of a vision-transformer block ------------------ */

/* The co-located ViT services (Sec. 3.1 MT; the ViT-B/16 mix) run, per encoder block, QKV projection ->
 * attention -> output projection -> FFN; the projections and the FFN are grouped dense forwards, and the two
 * calls below are what lies between them, each for all services in one launch (bf16 in and out, fp32
 * arithmetic).  Neither allocates nor synchronises. */

/* Rows of one service through a residual connection and a layer normalisation (Ba et al. 2016; the pre-norm
 * block of Dosovitskiy et al. 2021): s = x + r per element (r absent: s = x), then per row of d values
 * mu = mean(s), var = mean((s - mu)^2), y = (s - mu) / sqrt(var + eps) * gamma + beta.  The statistics and y
 * come from the unrounded fp32 sum; S receives the sum rounded to bf16.  64 bytes, the same on host and device. */
typedef struct {
    const void*  X;          /* device, bf16 [M, d] row-major, 16-byte aligned */
    const void*  R;          /* device, bf16 [M, d], or NULL */
    const float* gamma;      /* device, fp32 [d], 16-byte aligned */
    const float* beta;       /* device, fp32 [d], 16-byte aligned */
    void*        S;          /* device, bf16 [M, d], or NULL (the sum is not kept); may be the same buffer as X or R */
    void*        Y;          /* device, bf16 [M, d]; may be the same buffer as X or R when S is not */
    int32_t      M, d;       /* M >= 0; d a multiple of 8, 8 <= d <= EPARA_NORM_MAX_D */
    float        eps;        /* >= 0 */
    int32_t      first_row;  /* rows of all earlier groups: the running sum of M */
} epara_norm_args;
#define EPARA_NORM_MAX_D 8192

/* One kernel on `stream`: a wave per row (the row stays in registers between the two passes over it, the next row's
 * loads are in flight meanwhile), rows of all groups in one grid; a row finds its group by bisection over first_row.  G = 0 or no rows enqueues nothing.
 * Errors (from h_args): ERR_NULL (an array missing; X, gamma, beta or Y NULL in a group with rows), ERR_SHAPE
 * (M < 0, d out of range or not a multiple of 8, eps negative or not finite, first_row not the running sum, more
 * than 2^31 - 1 rows in all), ERR_ALIGN (X, R, S, Y, gamma or beta not 16-byte aligned). */
int32_t epara_add_layernorm(const epara_norm_args* h_args, const epara_norm_args* d_args, int32_t G, void* stream);

/* Scaled dot-product attention (Vaswani et al. 2017) of one service: its M = images * tokens rows are the output
 * of the QKV projection, a row = [Q | K | V] with each third d = heads * head_dim wide; per image and head,
 * S = Q K^T / sqrt(head_dim), P = softmax over the keys of every query row, O = P V, heads side by side in O.
 * The products run on the matrix cores (bf16 operands, fp32 sums); the softmax is fp32 with the row maximum
 * taken out; P is rounded to bf16 for the second product and the row sums divide its result.
 * 40 bytes, the same on host and device. */
typedef struct {
    const void* QKV;         /* device, bf16 [M, 3 * heads * head_dim] row-major, 16-byte aligned */
    void*       O;           /* device, bf16 [M, heads * head_dim], 16-byte aligned; not QKV */
    int32_t     M;           /* >= 0, a multiple of tokens */
    int32_t     tokens;      /* 1 .. EPARA_ATTN_MAX_TOKENS */
    int32_t     heads;       /* >= 1 */
    int32_t     head_dim;    /* EPARA_ATTN_HEAD_DIM */
    int32_t     first_item;  /* (image, head) pairs of all earlier groups: the running sum of (M / tokens) * heads */
    int32_t     reserved;
} epara_attn_args;
#define EPARA_ATTN_MAX_TOKENS 224
#define EPARA_ATTN_HEAD_DIM 64

/* One kernel on `stream` (compiled for 2, 4, 8 and 14 blocks of 16 keys; the longest image of the launch chooses):
 * a workgroup per (image, head) keeps that head's keys and (transposed) values in the LDS; its eight waves take the
 * query rows in blocks of 16.  G = 0 or no rows enqueues nothing.
 * Errors (from h_args): ERR_NULL; ERR_SHAPE (M < 0 or not a multiple of tokens, tokens or head_dim out of range,
 * heads < 1, O the same buffer as QKV, first_item not the running sum, more than 2^31 - 1 items); ERR_ALIGN (QKV or O
 * not 16-byte aligned). */
int32_t epara_attention(const epara_attn_args* h_args, const epara_attn_args* d_args, int32_t G, void* stream);

const char* epara_status_string(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* EPARA_H */
