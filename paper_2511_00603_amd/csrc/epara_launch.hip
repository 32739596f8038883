// Host side of the device entry points of libepara: validation of a launch against the planner's
// rules, then the kernels of the other translation units.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <cstring>
#include <mutex>
#include <vector>

#include "epara.h"
#include "epara_internal.h"

namespace {

constexpr int N_STREAM_CLASSES = 3;
constexpr int CHAIN_HEADER_WORDS = 4;     // error flag, exit count (the kernels use the same layout)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int64_t dtype_bytes(int32_t dtype) { return dtype == EPARA_F32 ? 4 : (dtype == EPARA_BF16 ? 2 : 1); }

// Every tile must be exactly what epara_plan_groups produces from one of the kernel class tables.
int32_t check_tiles(const epara_launch* L, int32_t in_dtype, int narrow)
{
    const bool f32 = in_dtype == EPARA_F32;
    epara_tile_class cls[2][4];
    int32_t ncls[2] = {0, 0}, nstream = 0;
    epara_kernel_classes(in_dtype, 0, narrow, cls[0], 4, &ncls[0], &nstream);
    if (!f32) epara_kernel_classes(in_dtype, 1, narrow, cls[1], 4, &ncls[1], &nstream);
    for (int64_t t = 0; t < L->n_tiles; ++t) {
        const epara_tile& tl = L->h_tiles[t];
        if (tl.group < 0 || tl.group >= L->G) return EPARA_ERR_SHAPE;
        const epara_group_args& a = L->h_args[tl.group];
        const int gated = a.act == EPARA_ACT_SWIGLU ? 1 : 0;
        if (tl.cls < 0 || tl.cls >= ncls[gated]) return EPARA_ERR_SHAPE;
        const epara_tile_class& c = cls[gated][tl.cls];
        if (a.M > c.max_M || (tl.cls > 0 && a.M <= cls[gated][tl.cls - 1].max_M)) return EPARA_ERR_SHAPE;
        if (tl.m0 < 0 || tl.n0 < 0 || tl.m0 >= a.M || tl.n0 >= a.N || tl.m0 % c.BM || tl.n0 % c.BN) return EPARA_ERR_SHAPE;
        const int32_t rows = a.M - tl.m0 < c.BM ? a.M - tl.m0 : c.BM;
        const int32_t cols = a.N - tl.n0 < c.BN ? a.N - tl.n0 : c.BN;
        if (tl.rows != rows || tl.cols != cols) return EPARA_ERR_SHAPE;
    }
    return EPARA_OK;
}

int32_t validate_launch(const epara_launch* L, int32_t in_dtype, int32_t out_dtype, int* narrow_out = nullptr)
{
    if (!L) return EPARA_ERR_NULL;
    const bool f32 = in_dtype == EPARA_F32;
    if (f32) { if (out_dtype != EPARA_F32) return EPARA_ERR_DTYPE; }
    else if (in_dtype == EPARA_BF16) { if (out_dtype != EPARA_BF16) return EPARA_ERR_DTYPE; }
    else if (in_dtype == EPARA_FP8_E4M3) { if (out_dtype != EPARA_BF16 && out_dtype != EPARA_FP8_E4M3) return EPARA_ERR_DTYPE; }
    else return EPARA_ERR_DTYPE;
    if (L->G < 0 || L->n_tiles < 0 || L->n_slots < 0) return EPARA_ERR_SHAPE;
    if (L->n_tiles == 0) return EPARA_OK;
    if (!L->h_args || !L->d_args || !L->h_tiles || !L->d_tiles || !L->d_order) return EPARA_ERR_NULL;
    if (L->n_workgroups <= 0 || L->n_slots < L->n_tiles || L->n_slots % L->n_workgroups != 0 || L->n_tiles > INT32_MAX)
        return EPARA_ERR_SHAPE;
    const int esz = f32 ? 4 : (in_dtype == EPARA_BF16 ? 2 : 1);
    for (int32_t g = 0; g < L->G; ++g) {
        const epara_group_args& a = L->h_args[g];
        if (a.M < 0 || a.K <= 0 || a.N <= 0) return EPARA_ERR_SHAPE;
        if (a.act < EPARA_ACT_NONE || a.act > EPARA_ACT_SWIGLU) return EPARA_ERR_DTYPE;
        if (a.act == EPARA_ACT_SWIGLU && (f32 || a.bias)) return EPARA_ERR_DTYPE;
        if (a.M == 0) continue;
        if (!a.X || !a.W || !a.Y || (a.act == EPARA_ACT_SWIGLU && !a.W2)) return EPARA_ERR_NULL;
        if (!aligned16(a.X) || !aligned16(a.W) || !aligned16(a.Y) || !aligned16(a.W2) || !aligned16(a.bias))
            return EPARA_ERR_ALIGN;
        if (!f32 && (static_cast<int64_t>(a.K) * esz) % 16 != 0) return EPARA_ERR_ALIGN;
        // the matrix-core kernels address a tile's operands with 32-bit byte offsets (256 rows, 16 column blocks)
        if (!f32 && static_cast<int64_t>(a.K) * esz > (1 << 23)) return EPARA_ERR_SHAPE;
    }
    // a launch is either all SwiGLU groups or none: the tile classes differ
    {
        int32_t n_gated = 0, n_live = 0;
        for (int32_t g = 0; g < L->G; ++g)
            if (L->h_args[g].M > 0) { ++n_live; n_gated += L->h_args[g].act == EPARA_ACT_SWIGLU; }
        if (n_gated != 0 && n_gated != n_live) return EPARA_ERR_DTYPE;
    }
    int32_t last = EPARA_OK, narrow = 0;
    for (; narrow < (f32 ? 1 : 2); ++narrow) {
        last = check_tiles(L, in_dtype, narrow);
        if (last == EPARA_OK) break;
    }
    if (last != EPARA_OK) return last;
    if (narrow_out) *narrow_out = narrow;
    // split tiles: the groups' slots and the counts must be the layout's, and the workspace must hold them
    if (L->n_split_tiles < 0 || L->n_panel_split_tiles < 0) return EPARA_ERR_SHAPE;
    if (L->n_split_tiles > 0 || L->n_panel_split_tiles > 0) {
        if (f32) return EPARA_ERR_DTYPE;
        int gated = 0;
        for (int32_t g = 0; g < L->G; ++g)
            if (L->h_args[g].M > 0 && L->h_args[g].act == EPARA_ACT_SWIGLU) gated = 1;
        epara_tile_class cls[4];
        int32_t ncls = 0, nstream = 0, n_split = 0, n_panel = 0, parts = 1, more = 0;
        int64_t bytes = 0;
        epara_kernel_classes(in_dtype, gated, narrow, cls, 4, &ncls, &nstream);
        std::vector<epara_group_desc> d(static_cast<size_t>(L->G));
        std::vector<int32_t> base(static_cast<size_t>(L->G));
        for (int32_t g = 0; g < L->G; ++g) d[g] = {L->h_args[g].M, L->h_args[g].K, L->h_args[g].N, L->h_args[g].act, 0, 0};
        if (int32_t st = epara_split_layout(d.data(), L->G, cls, ncls, nstream, base.data(), &n_split, &bytes)) return st;
        if (int32_t st = epara_panel_split(d.data(), L->G, cls, ncls, nstream, L->n_workgroups, &n_panel, &parts, &more)) return st;
        if (n_split != L->n_split_tiles || n_panel != L->n_panel_split_tiles) return EPARA_ERR_SHAPE;
        for (int32_t g = 0; g < L->G; ++g)
            if (base[g] >= 0 && L->h_args[g].reserved != base[g]) return EPARA_ERR_SHAPE;
        if (!L->d_workspace) return EPARA_ERR_NULL;
        if (reinterpret_cast<uintptr_t>(L->d_workspace) % 256 != 0) return EPARA_ERR_ALIGN;
        if (L->workspace_bytes < epara_split_workspace_bytes(n_split, n_panel)) return EPARA_ERR_CAPACITY;
    }
    return EPARA_OK;
}

int32_t enqueue(const epara_launch* L, int32_t in_dtype, int32_t out_dtype, int narrow, hipStream_t stream)
{
    if (L->n_tiles == 0) return EPARA_OK;
    int gated = 0;
    for (int32_t g = 0; g < L->G; ++g)
        if (L->h_args[g].M > 0 && L->h_args[g].act == EPARA_ACT_SWIGLU) gated = 1;
    int panel_only = 1;                       // launches without streaming tiles run a kernel without that code
    for (int64_t t = 0; t < L->n_tiles; ++t)
        if (L->h_tiles[t].cls < N_STREAM_CLASSES) { panel_only = 0; break; }
    const unsigned grid = static_cast<unsigned>(L->n_workgroups);
    const long n_slots = static_cast<long>(L->n_slots);
    (void)hipGetLastError();
    hipError_t e;
    if (in_dtype == EPARA_F32)       e = epara_enqueue_f32(grid, stream, L->d_args, L->d_tiles, L->d_order, n_slots);
    else if (in_dtype == EPARA_BF16) e = (gated ? epara_enqueue_bf16_gated : epara_enqueue_bf16_plain)(panel_only, grid, stream, L->d_args, L->d_tiles, L->d_order, n_slots, out_dtype, narrow, static_cast<uint32_t*>(L->d_workspace), L->n_split_tiles, L->n_panel_split_tiles, static_cast<int>(L->n_tiles - L->n_panel_split_tiles));
    else                             e = (gated ? epara_enqueue_fp8_gated : epara_enqueue_fp8_plain)(panel_only, grid, stream, L->d_args, L->d_tiles, L->d_order, n_slots, out_dtype, narrow, static_cast<uint32_t*>(L->d_workspace), L->n_split_tiles, L->n_panel_split_tiles, static_cast<int>(L->n_tiles - L->n_panel_split_tiles));
    return e == hipSuccess ? EPARA_OK : EPARA_ERR_HIP;
}

}  // namespace

extern "C" {

int64_t epara_packed_weight_bytes(int32_t K, int32_t N, int32_t dtype)
{
    if (K <= 0 || N <= 0) return -1;
    if (dtype == EPARA_F32) return static_cast<int64_t>(K) * N * 4;
    if (dtype != EPARA_BF16 && dtype != EPARA_FP8_E4M3) return -1;
    const int64_t KF = dtype == EPARA_BF16 ? 32 : 64;
    const int64_t stages = ((K + KF - 1) / KF + 3) / 4 * 4;        // padded to a multiple of four (zeros)
    return ((static_cast<int64_t>(N) + 15) / 16) * stages * 1024;
}

int32_t epara_pack_weights(const void* d_W, int32_t K, int32_t N, int32_t dtype,
                           void* d_packed, int64_t packed_bytes, void* stream)
{
    if (!d_W || !d_packed) return EPARA_ERR_NULL;
    if (K <= 0 || N <= 0) return EPARA_ERR_SHAPE;
    const int64_t need = epara_packed_weight_bytes(K, N, dtype);
    if (need < 0) return EPARA_ERR_DTYPE;
    if (packed_bytes < need) return EPARA_ERR_CAPACITY;
    if (!aligned16(d_packed)) return EPARA_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    (void)hipGetLastError();
    if (dtype == EPARA_F32) {
        if (hipMemcpyAsync(d_packed, d_W, static_cast<size_t>(need), hipMemcpyDeviceToDevice, st) != hipSuccess)
            return EPARA_ERR_HIP;
        return EPARA_OK;
    }
    const hipError_t e = epara_enqueue_pack(dtype == EPARA_BF16 ? 2 : 1, static_cast<const char*>(d_W), K, N,
                                            static_cast<char*>(d_packed), need / 16, st);
    return e == hipSuccess ? EPARA_OK : EPARA_ERR_HIP;
}

int32_t epara_grouped_forward(const epara_launch* launch, int32_t in_dtype, int32_t out_dtype, void* stream)
{
    int narrow = 0;
    if (int32_t st = validate_launch(launch, in_dtype, out_dtype, &narrow)) return st;
    return enqueue(launch, in_dtype, out_dtype, narrow, static_cast<hipStream_t>(stream));
}

int32_t epara_grouped_ffn_swiglu(const epara_launch* up, const epara_launch* down,
                                 int32_t in_dtype, int32_t h_dtype, int32_t out_dtype, void* stream)
{
    if (!up || !down) return EPARA_ERR_NULL;
    if (in_dtype == EPARA_BF16) { if (h_dtype != EPARA_BF16 || out_dtype != EPARA_BF16) return EPARA_ERR_DTYPE; }
    else if (in_dtype == EPARA_FP8_E4M3) { if (h_dtype != EPARA_FP8_E4M3 || out_dtype != EPARA_BF16) return EPARA_ERR_DTYPE; }
    else return EPARA_ERR_DTYPE;
    int narrow_up = 0, narrow_down = 0;
    if (int32_t st = validate_launch(up, in_dtype, h_dtype, &narrow_up)) return st;
    if (int32_t st = validate_launch(down, in_dtype, out_dtype, &narrow_down)) return st;
    if (up->G != down->G) return EPARA_ERR_SHAPE;
    if (up->n_tiles > 0 || down->n_tiles > 0) {
        for (int32_t g = 0; g < up->G; ++g) {
            const epara_group_args& u = up->h_args[g];
            const epara_group_args& d = down->h_args[g];
            if (u.act != EPARA_ACT_SWIGLU || d.act != EPARA_ACT_NONE) return EPARA_ERR_DTYPE;
            if (u.M != d.M || u.N != d.K || u.K != d.N || u.Y != d.X) return EPARA_ERR_SHAPE;
        }
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (int32_t rc = enqueue(up, in_dtype, h_dtype, narrow_up, st)) return rc;
    return enqueue(down, in_dtype, out_dtype, narrow_down, st);
}

int64_t epara_chain_workspace_bytes(int32_t n_counters)
{
    if (n_counters < 0) return -1;
    return ((static_cast<int64_t>(CHAIN_HEADER_WORDS) + n_counters) * 4 + 255) / 256 * 256;
}

int32_t epara_chain_workspace_init(void* d_workspace, int64_t bytes, void* stream)
{
    if (!d_workspace) return EPARA_ERR_NULL;
    if (bytes < 16 || bytes % 4) return EPARA_ERR_SHAPE;
    if (!aligned16(d_workspace)) return EPARA_ERR_ALIGN;
    (void)hipGetLastError();
    const hipError_t e = epara_enqueue_fill_words(static_cast<uint32_t*>(d_workspace), bytes / 4, 0u, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? EPARA_OK : EPARA_ERR_HIP;
}

// n_counters_out: when given, only validates and reports the number of counters the chain needs.
static int32_t chain_impl(const epara_chain_phase* phases, int32_t n_phases, int32_t in_dtype,
                          void* d_workspace, int64_t workspace_bytes, uint32_t spin_limit, void* stream, int32_t* n_counters_out)
{
    if (!phases || (!d_workspace && !n_counters_out)) return EPARA_ERR_NULL;
    if (n_phases < 1 || n_phases > EPARA_MAX_CHAIN_PHASES) return EPARA_ERR_SHAPE;
    if (d_workspace && !aligned16(d_workspace)) return EPARA_ERR_ALIGN;
    epara_chain_scalars S;
    std::memset(&S, 0, sizeof S);
    const epara_group_args* d_args[EPARA_MAX_CHAIN_PHASES] = {};
    const epara_tile* d_tiles[EPARA_MAX_CHAIN_PHASES] = {};
    const int32_t* d_order[EPARA_MAX_CHAIN_PHASES] = {};
    const epara_chain_wait* d_waits[EPARA_MAX_CHAIN_PHASES] = {};
    int gated[EPARA_MAX_CHAIN_PHASES] = {};
    int32_t n_counters = 0, n_workgroups = 0;
    bool any = false;
    struct span { uintptr_t at; int64_t bytes; };
    std::vector<span> produced;               // the tensors some group waits for
    for (int32_t p = 0; p < n_phases; ++p) {
        const epara_chain_phase& ph = phases[p];
        const epara_launch* L = ph.launch;
        int narrow = 0;
        if (int32_t st = validate_launch(L, in_dtype, ph.out_dtype, &narrow)) return st;
        if (L->n_split_tiles != 0 || L->n_panel_split_tiles != 0) return EPARA_ERR_SHAPE;   // the phases of a chain are scheduled without splitting K
        if (ph.counter_base < 0 || ph.counter_base > INT32_MAX - L->G) return EPARA_ERR_SHAPE;
        for (int32_t q = 0; q < p; ++q)       // counter ranges must not overlap
            if (ph.counter_base < phases[q].counter_base + phases[q].launch->G &&
                phases[q].counter_base < ph.counter_base + L->G) return EPARA_ERR_SHAPE;
        n_counters = std::max(n_counters, ph.counter_base + L->G);
        if (L->n_tiles > 0) {
            if (any && L->n_workgroups != n_workgroups) return EPARA_ERR_SHAPE;
            n_workgroups = L->n_workgroups;
            any = true;
        }
        for (int32_t g = 0; g < L->G && L->n_tiles > 0; ++g)
            if (L->h_args[g].M > 0 && L->h_args[g].act == EPARA_ACT_SWIGLU) gated[p] = 1;
        if (ph.h_waits && L->n_tiles > 0) {
            if (p == 0) return EPARA_ERR_SHAPE;
            if (!ph.d_waits) return EPARA_ERR_NULL;
            const epara_chain_phase& prev = phases[p - 1];
            const epara_launch* Lp = prev.launch;
            std::vector<int64_t> count(static_cast<size_t>(Lp->G), 0);
            for (int64_t t = 0; t < Lp->n_tiles; ++t) ++count[Lp->h_tiles[t].group];
            if (prev.out_dtype != in_dtype) return EPARA_ERR_DTYPE;          // the phase reads what the one before stored
            for (int32_t g = 0; g < L->G; ++g) {
                const epara_chain_wait& w = ph.h_waits[g];
                if (w.counter < 0) continue;
                const int32_t q = w.counter - prev.counter_base;
                if (q < 0 || q >= Lp->G || w.need != count[q]) return EPARA_ERR_SHAPE;
                const epara_group_args& a = L->h_args[g];
                if (a.M == 0) continue;
                if (Lp->n_tiles == 0) return EPARA_ERR_SHAPE;
                const epara_group_args& b = Lp->h_args[q];
                if (a.X != b.Y || a.M != b.M || a.K != b.N) return EPARA_ERR_SHAPE;
                produced.push_back({reinterpret_cast<uintptr_t>(b.Y), static_cast<int64_t>(b.M) * b.N * dtype_bytes(prev.out_dtype)});
            }
            d_waits[p] = ph.d_waits;
        }
        d_args[p] = L->d_args; d_tiles[p] = L->d_tiles; d_order[p] = L->d_order;
        S.n_slots[p] = L->n_tiles > 0 ? L->n_slots : 0;
        S.out_dtype[p] = ph.out_dtype; S.narrow[p] = narrow; S.counter_base[p] = ph.counter_base;
    }
    // A produced tensor must own its cache lines: a consumer invalidates nothing after its wait, so a line
    // that also holds bytes of another tensor of the chain could be cached (by a read of that tensor)
    // before the produced tensor was written.  It must start on a line and nothing else may begin in
    // the rest of its last line.
    for (const span& y : produced) {
        if (y.at % 128 != 0) return EPARA_ERR_ALIGN;
        const uintptr_t end = y.at + static_cast<uintptr_t>(y.bytes), line_end = (end + 127) / 128 * 128;
        for (int32_t p = 0; p < n_phases; ++p) {
            const epara_launch* L = phases[p].launch;
            for (int32_t g = 0; g < L->G && L->n_tiles > 0; ++g) {
                const epara_group_args& a = L->h_args[g];
                if (a.M == 0) continue;
                const span others[5] = {
                    {reinterpret_cast<uintptr_t>(a.X), static_cast<int64_t>(a.M) * a.K * dtype_bytes(in_dtype)},
                    {reinterpret_cast<uintptr_t>(a.Y), static_cast<int64_t>(a.M) * a.N * dtype_bytes(phases[p].out_dtype)},
                    {reinterpret_cast<uintptr_t>(a.W), epara_packed_weight_bytes(a.K, a.N, in_dtype)},
                    {reinterpret_cast<uintptr_t>(a.W2), a.W2 ? epara_packed_weight_bytes(a.K, a.N, in_dtype) : 0},
                    {reinterpret_cast<uintptr_t>(a.bias), a.bias ? static_cast<int64_t>(a.N) * 4 : 0}};
                for (const span& o : others) {
                    if (o.bytes <= 0 || o.at == y.at) continue;
                    if (o.at < line_end && o.at + static_cast<uintptr_t>(o.bytes) > end) return EPARA_ERR_ALIGN;
                }
            }
        }
    }
    // the kernels exist for chains without gating and for the two phases of a SwiGLU FFN
    bool ffn = false;
    for (int32_t p = 0; p < n_phases; ++p) ffn = ffn || gated[p];
    if (ffn && !(n_phases == 2 && gated[0] && !gated[1])) return EPARA_ERR_DTYPE;
    if (n_counters_out) { *n_counters_out = n_counters; return EPARA_OK; }
    if (workspace_bytes < epara_chain_workspace_bytes(n_counters)) return EPARA_ERR_CAPACITY;
    if (!any) return EPARA_OK;
    S.ws = static_cast<uint32_t*>(d_workspace);
    S.spin_limit = spin_limit ? spin_limit : (1u << 20);
    S.n_phases = n_phases;
    S.n_counters = n_counters;

    hipStream_t st = static_cast<hipStream_t>(stream);
    typedef hipError_t (*entry_t)(const epara_chain_tables&, const epara_chain_scalars&, unsigned, hipStream_t, int64_t*);
    entry_t fn = in_dtype == EPARA_F32 ? epara_chain_f32
               : in_dtype == EPARA_BF16 ? (ffn ? epara_chain_bf16_ffn : epara_chain_bf16_plain)
                                        : (ffn ? epara_chain_fp8_ffn : epara_chain_fp8_plain);
    epara_chain_tables T;
    for (int p = 0; p < EPARA_MAX_CHAIN_PHASES; ++p) { T.args[p] = d_args[p]; T.tiles[p] = d_tiles[p]; T.order[p] = d_order[p]; T.waits[p] = d_waits[p]; }
    (void)hipGetLastError();
    // a waiting workgroup must not keep the one it waits for off the GPU: the whole grid has to be resident
    struct limit { int dev; entry_t fn; int64_t resident; };
    static thread_local limit cache[8] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return EPARA_ERR_HIP;
    int64_t resident = -1;
    for (const limit& l : cache)
        if (l.fn == fn && l.dev == dev) resident = l.resident;
    if (resident < 0) {
        if (fn(T, S, 0, st, &resident) != hipSuccess) return EPARA_ERR_HIP;
        static thread_local int next = 0;
        cache[next++ % 8] = {dev, fn, resident};
    }
    if (static_cast<int64_t>(n_workgroups) > resident) return EPARA_ERR_SHAPE;
    return fn(T, S, static_cast<unsigned>(n_workgroups), st, nullptr) == hipSuccess ? EPARA_OK : EPARA_ERR_HIP;
}

int32_t epara_workspace_init(void* d_workspace, int64_t bytes, void* stream)
{
    return epara_chain_workspace_init(d_workspace, bytes, stream);
}

int32_t epara_grouped_chain(const epara_chain_phase* phases, int32_t n_phases, int32_t in_dtype,
                            void* d_workspace, int64_t workspace_bytes, uint32_t spin_limit, void* stream)
{
    return chain_impl(phases, n_phases, in_dtype, d_workspace, workspace_bytes, spin_limit, stream, nullptr);
}

// ---- the same chain on the library's own scratch (for callers that cannot allocate)
//
// The completion counters live in a file-scope device array.  Its name is only a host-side stand-in:
// the address of each GPU's own copy is looked up once per device (with that device current) and kept.
static __device__ __align__(256) uint32_t scratch[CHAIN_HEADER_WORDS + EPARA_STATIC_CHAIN_COUNTERS];

static int32_t scratch_address(uint32_t** out)
{
    constexpr int MAX_DEVICES = 64;
    static std::mutex lock;
    static uint32_t* address[MAX_DEVICES] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return EPARA_ERR_HIP;
    std::lock_guard<std::mutex> guard(lock);
    if (!address[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return EPARA_ERR_HIP;
        address[dev] = static_cast<uint32_t*>(p);
    }
    *out = address[dev];
    return EPARA_OK;
}

int32_t epara_grouped_chain_static(const epara_chain_phase* phases, int32_t n_phases, int32_t in_dtype,
                                   uint32_t spin_limit, int32_t* d_flag, void* stream)
{
    int32_t n_counters = 0;
    if (int32_t st = chain_impl(phases, n_phases, in_dtype, nullptr, 0, spin_limit, stream, &n_counters)) return st;
    if (n_counters > EPARA_STATIC_CHAIN_COUNTERS) return EPARA_ERR_CAPACITY;
    if (d_flag && (reinterpret_cast<uintptr_t>(d_flag) & 3u)) return EPARA_ERR_ALIGN;
    uint32_t* ws = nullptr;
    if (int32_t st = scratch_address(&ws)) return st;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    (void)hipGetLastError();
    // the array keeps what the last call left (an error flag of a wait that ran out): start from zero
    const long words = CHAIN_HEADER_WORDS + n_counters;
    if (epara_enqueue_fill_words(ws, words, 0u, hs) != hipSuccess) return EPARA_ERR_HIP;
    if (int32_t st = chain_impl(phases, n_phases, in_dtype, ws, epara_chain_workspace_bytes(EPARA_STATIC_CHAIN_COUNTERS), spin_limit, stream, nullptr))
        return st;
    if (d_flag && epara_enqueue_copy_word(ws, reinterpret_cast<uint32_t*>(d_flag), hs) != hipSuccess) return EPARA_ERR_HIP;
    return EPARA_OK;
}

int32_t epara_chain_status(void* d_workspace, void* stream, int32_t* flag)
{
    if (!d_workspace || !flag) return EPARA_ERR_NULL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint32_t v = 0;
    if (hipStreamSynchronize(st) != hipSuccess) return EPARA_ERR_HIP;
    if (hipMemcpy(&v, d_workspace, 4, hipMemcpyDeviceToHost) != hipSuccess) return EPARA_ERR_HIP;
    *flag = static_cast<int32_t>(v);
    if (v) {
        const uint32_t zero = 0;
        if (hipMemcpy(d_workspace, &zero, 4, hipMemcpyHostToDevice) != hipSuccess) return EPARA_ERR_HIP;
    }
    return EPARA_OK;
}

}  // extern "C"
