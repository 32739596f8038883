// The persistent kernels of libepara for bf16 / fp8 inputs: one launch serves every co-located
// service (the MT operator of Sec. 3.1).  Persistent workgroups walk a device tile table in a
// precomputed visit order; a tile is either a panel tile (epara_panel.h: 256 rows, matrix-core
// bound) or a streaming tile (epara_stream.h: a whole batch of at most 64 rows against weights
// streamed from HBM).  Bias, activation, SwiGLU gating, fp8 scales and the output cast are fused in
// the epilogues.  A workgroup is four waves, one per SIMD, so a wave may use the whole 512-entry
// register file.
#ifndef EPARA_GROUPED_H
#define EPARA_GROUPED_H

#include "epara_device.h"
#include "epara_internal.h"
#include "epara_panel.h"
#include "epara_stream.h"

namespace {

// Streaming classes: (row blocks, weight column blocks, ring depth) = (1, 2, 4), (2, 4, 3) and
// (4, 8, 2) or, in a launch planned with the narrow table, (4, 4, 3).  PANEL_ONLY: the launch holds
// no streaming tile (checked on the host), so the kernel carries no code for them.
// Counts the workgroup's visits to split tiles at the tiles' counters (one atomic instruction for all of
// them) and finishes the tiles at which it arrived last.  Every partial sum of the workgroup is in memory
// before the count says so; whoever finishes a tile puts its counter back to zero for the next launch.
template <int DT, bool GATED, bool PANEL_ONLY>
__device__ __forceinline__ void split_flush(const epara_group_args* __restrict__ args, const epara_tile* __restrict__ tiles,
                                            int out_dtype, int narrow, char* lds, const split_ctx* sp, split_pending& pend)
{
    if (pend.count == 0) return;
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    wait_vmcnt<0>();
    __syncthreads();
    __attribute__((address_space(3))) uint32_t* box = (__attribute__((address_space(3))) uint32_t*)(ldsptr)lds;
    if (wave == 0) {
        const bool mine = lane < pend.count;
        uint32_t before = 0;
        if (mine) before = __hip_atomic_fetch_add(sp->ws + (pend.slots & 0xFFFFFFF), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long last = __ballot(mine && before == (static_cast<uint32_t>(pend.slots) >> 28));
        if (lane == 0) { box[0] = static_cast<uint32_t>(last); box[1] = static_cast<uint32_t>(last >> 32); }
    }
    __syncthreads();
    unsigned long long last = (static_cast<unsigned long long>(box[1]) << 32) | box[0];
    last = (static_cast<unsigned long long>(__builtin_amdgcn_readfirstlane(static_cast<int>(last >> 32))) << 32) |
           static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(last)));
    __syncthreads();                                             // the box's place in LDS is free again
    while (last) {
        const int i = __builtin_ctzll(last);
        last &= last - 1;
        const int entry = __builtin_amdgcn_readlane(pend.entries, i);
        const int info = __builtin_amdgcn_readlane(pend.slots, i);
        const int slot = info & 0xFFFFFFF, nparts = (static_cast<uint32_t>(info) >> 28) + 1;
        const epara_tile tl = tiles[order_tile(entry)];
        const epara_group_args ga = args[tl.group];
        if (tl.cls >= N_STREAM_CLASSES) {
            if constexpr (!GATED) panel_split_finish<DT>(ga, tl, out_dtype, slot - sp->n_split, nparts, tid, sp, lds);
        } else if constexpr (!PANEL_ONLY) {
            if (tl.cls == 1)                 split_finish<DT, GATED, 2, 4>(ga, out_dtype, tl.n0, tl.cols, slot, nparts, wave, lane, lds, sp);
            else if (tl.cls == 2 && !narrow) split_finish<DT, GATED, 4, 8>(ga, out_dtype, tl.n0, tl.cols, slot, nparts, wave, lane, lds, sp);
            else if (tl.cls == 2)            split_finish<DT, GATED, 4, 4>(ga, out_dtype, tl.n0, tl.cols, slot, nparts, wave, lane, lds, sp);
        }
        if (tid == 0) __hip_atomic_store(sp->ws + slot, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();                                         // the next tile's parts land where these were read
    }
    pend.count = 0;
}

template <int DT, bool GATED, bool CHAIN, bool PANEL_ONLY>
__device__ __forceinline__ void grouped_body(const epara_group_args* __restrict__ args, const epara_tile* __restrict__ tiles,
                                             const int32_t* __restrict__ order, long n_slots, int out_dtype, int narrow, char* lds,
                                             chain_ctx* chain = nullptr, const split_ctx* sp = nullptr)
{
    // which kernels can meet tiles visited in parts of K: bf16 only, streaming tiles and plain panel tiles of single launches
    constexpr bool HAS_SPLIT = !CHAIN && DT == EPARA_BF16 && (!PANEL_ONLY || !GATED);
    const long stride = gridDim.x;
    long s = blockIdx.x;
    split_pending pend = {0, 0, 0};
    run_next nx = {};
    while (s < n_slots) {
        int t;
        epara_tile tl;
        const bool known = nx.known;                             // the run before has read this slot already
        if (known) { t = nx.entry; tl = nx.tl; }
        else {
            t = order[s];
            if (t < 0) { s += stride; continue; }
            tl = tiles[order_tile(t)];
        }
        nx.known = false;
        if constexpr (CHAIN) chain_wait(*chain, tl.group);
        if constexpr (HAS_SPLIT) { if (pend.count >= 63) split_flush<DT, GATED, PANEL_ONLY>(args, tiles, out_dtype, narrow, lds, sp, pend); }
        if constexpr (!PANEL_ONLY) {
            const epara_group_args ga0 = nx.ga;
            if (tl.cls == 0)      { s = skinny_run<DT, GATED, CHAIN, 0, 1, 2, 4>(args, tiles, order, s, t, tl, ga0, known, n_slots, stride, out_dtype, lds, chain, sp, &pend, nx); continue; }
            else if (tl.cls == 1) { s = skinny_run<DT, GATED, CHAIN, 1, 2, 4, 3>(args, tiles, order, s, t, tl, ga0, known, n_slots, stride, out_dtype, lds, chain, sp, &pend, nx); continue; }
            else if (tl.cls == 2 && !narrow) { s = skinny_run<DT, GATED, CHAIN, 2, 4, 8, 2>(args, tiles, order, s, t, tl, ga0, known, n_slots, stride, out_dtype, lds, chain, sp, &pend, nx); continue; }
            else if (tl.cls == 2) { s = skinny_run<DT, GATED, CHAIN, 2, 4, 4, 3>(args, tiles, order, s, t, tl, ga0, known, n_slots, stride, out_dtype, lds, chain, sp, &pend, nx); continue; }
        }
        s = panel_run<DT, GATED, CHAIN, CHAIN>(args, tiles, order, s, n_slots, stride, out_dtype, lds, chain, sp, &pend);
        nx = run_next{};                                         // nothing is carried across a panel run
    }
    if constexpr (HAS_SPLIT) split_flush<DT, GATED, PANEL_ONLY>(args, tiles, out_dtype, narrow, lds, sp, pend);
}

template <int DT, bool GATED, bool PANEL_ONLY>
__global__ __launch_bounds__(NT) void grouped_kernel(const epara_group_args* __restrict__ args,
                                                     const epara_tile* __restrict__ tiles,
                                                     const int32_t* __restrict__ order,
                                                     long n_slots, int out_dtype, int narrow, uint32_t* split_ws, int n_split, int n_panel_split, int first_panel_split)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const split_ctx sp = {split_ws, n_split, n_panel_split, first_panel_split};
    grouped_body<DT, GATED, false, PANEL_ONLY>(args, tiles, order, n_slots, out_dtype, narrow, lds, nullptr, &sp);
}

template <int DT, bool GATED>
hipError_t enqueue_grouped(int panel_only, unsigned grid, hipStream_t stream, const epara_group_args* args, const epara_tile* tiles,
                           const int32_t* order, long n_slots, int out_dtype, int narrow, uint32_t* split_ws, int n_split, int n_panel_split, int first_panel_split)
{
    static const hipError_t attr0 = hipFuncSetAttribute(reinterpret_cast<const void*>(&grouped_kernel<DT, GATED, false>),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    static const hipError_t attr1 = hipFuncSetAttribute(reinterpret_cast<const void*>(&grouped_kernel<DT, GATED, true>),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (attr0 != hipSuccess) return attr0;
    if (attr1 != hipSuccess) return attr1;
    if (panel_only)
        hipLaunchKernelGGL((grouped_kernel<DT, GATED, true>), dim3(grid), dim3(NT), LDS_BYTES, stream, args, tiles, order, n_slots, out_dtype, narrow, split_ws, n_split, n_panel_split, first_panel_split);
    else
        hipLaunchKernelGGL((grouped_kernel<DT, GATED, false>), dim3(grid), dim3(NT), LDS_BYTES, stream, args, tiles, order, n_slots, out_dtype, narrow, split_ws, n_split, n_panel_split, first_panel_split);
    return hipGetLastError();
}

// ---- a chain of launches as one kernel: the phases one after the other in every workgroup
//
// The tables of every phase are kernel arguments of their own (not fields of a structure in memory):
// only then does the compiler know them as read-only global memory that nothing in the kernel
// writes, and fetch tile, order and argument records with scalar loads as in the single-launch
// kernel -- the streaming pipeline counts its outstanding vector loads and has no room for others.
#define CHAIN_TABLES(i) const epara_group_args* __restrict__ a##i, const epara_tile* __restrict__ t##i, \
                        const int32_t* __restrict__ o##i, const epara_chain_wait* __restrict__ w##i
#define CHAIN_PICK(p, x) ((p) == 0 ? x##0 : (p) == 1 ? x##1 : (p) == 2 ? x##2 : x##3)

__device__ __forceinline__ chain_ctx chain_begin(const epara_chain_scalars& S)
{
    chain_ctx c;
    c.waits = nullptr; c.ws = S.ws; c.spin_limit = S.spin_limit; c.counter_base = 0;
    c.pend_group[0] = c.pend_group[1] = -1; c.pend_n[0] = c.pend_n[1] = 0; c.ok_group = -1;
    return c;
}

__device__ __forceinline__ void chain_enter_phase(chain_ctx& c, const epara_chain_wait* waits, int counter_base)
{
    chain_flush(c);                          // counts of the phase before go to that phase's counters
    c.waits = waits;
    c.counter_base = counter_base;
    c.ok_group = -1;
}

// FFN: exactly two phases, SwiGLU gate/up then down.  Otherwise: up to four phases without gating.
template <int DT, bool FFN>
__global__ __launch_bounds__(NT) void grouped_chain_kernel(CHAIN_TABLES(0), CHAIN_TABLES(1), CHAIN_TABLES(2), CHAIN_TABLES(3),
                                                           const epara_chain_scalars S)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    chain_ctx c = chain_begin(S);
    if constexpr (FFN) {
        chain_enter_phase(c, nullptr, S.counter_base[0]);
        grouped_body<DT, true, true, false>(a0, t0, o0, S.n_slots[0], S.out_dtype[0], S.narrow[0], lds, &c);
        chain_enter_phase(c, w1, S.counter_base[1]);
        grouped_body<DT, false, true, false>(a1, t1, o1, S.n_slots[1], S.out_dtype[1], S.narrow[1], lds, &c);
    } else {
        for (int p = 0; p < S.n_phases; ++p) {
            chain_enter_phase(c, CHAIN_PICK(p, w), S.counter_base[p]);
            grouped_body<DT, false, true, false>(CHAIN_PICK(p, a), CHAIN_PICK(p, t), CHAIN_PICK(p, o), S.n_slots[p], S.out_dtype[p],
                                                 S.narrow[p], lds, &c);
        }
    }
    chain_exit(c, S.n_counters);
}

template <int DT, bool FFN>
hipError_t chain_kernel_entry(const epara_chain_tables& T, const epara_chain_scalars& S, unsigned grid, hipStream_t stream, int64_t* resident)
{
    const void* fn = reinterpret_cast<const void*>(&grouped_chain_kernel<DT, FFN>);
    static const hipError_t attr = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (attr != hipSuccess) return attr;
    if (resident) {                          // how many workgroups of this kernel the current device holds at once
        int per_cu = 0, cus = 0, dev = 0;
        if (hipError_t e = hipGetDevice(&dev)) return e;
        if (hipError_t e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) return e;
        if (hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, NT, LDS_BYTES)) return e;
        *resident = static_cast<int64_t>(per_cu) * cus;
        return hipSuccess;
    }
    hipLaunchKernelGGL((grouped_chain_kernel<DT, FFN>), dim3(grid), dim3(NT), LDS_BYTES, stream,
                       T.args[0], T.tiles[0], T.order[0], T.waits[0], T.args[1], T.tiles[1], T.order[1], T.waits[1],
                       T.args[2], T.tiles[2], T.order[2], T.waits[2], T.args[3], T.tiles[3], T.order[3], T.waits[3], S);
    return hipGetLastError();
}

}  // namespace

#endif
