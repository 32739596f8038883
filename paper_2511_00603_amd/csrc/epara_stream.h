// Streaming tiles of libepara: small batches against weights streamed from HBM.
#ifndef EPARA_STREAM_H
#define EPARA_STREAM_H

#include "epara_device.h"

namespace {

// ------------------------------------------------------------------ skinny tiles (weight streaming)

// Small batches are bandwidth bound: the weights are streamed from HBM exactly once, straight
// into MFMA operand registers (each load instruction of a wave reads 1 KiB of consecutive packed
// weights), while the activations are re-read from L2 by every tile, through a small LDS ring per
// wave (see skinny_setup).  To keep that re-read at half the weight traffic, a tile of streaming
// class c = 0, 1, 2 pairs MB = 1, 2, 4 blocks of 16 rows (the whole batch) with NFR = 2, 4, 8
// weight column blocks: 32 / 64 / 128 output columns, or for gated groups NFR/2 gate blocks and
// the matching NFR/2 up blocks (16 / 32 / 64 hidden columns).  K is walked in steps of two packed
// fragments (128 bytes of every activation row, so a row's cache line is used whole); wave w takes
// a contiguous quarter of the steps (a wave then reads one sequential stream per column block, which
// the memory system serves faster than four waves interleaving 2-KiB pieces).  The four partial sums
// meet in LDS and are added in wave order: the result does not depend on timing.
//
// Consecutive tiles of one class that a workgroup owns are processed as one software-pipelined
// stream: a ring of U slots per wave (weights in registers, activations in LDS) stays full across
// tile boundaries, so the loads of the next tile are in flight while this tile is reduced and
// stored; the last tile of a run drains the ring.  Every tile is padded to a whole number of U
// steps; padding steps, rows past the batch and column blocks past N re-load a valid address and
// are not multiplied / not stored.  The scheduling barriers keep the compiler from sinking the
// prefetch loads down to their first use.
template <int NFR>
struct skinny_tile_state {
    gcptr w[NFR];          // uniform: start of each weight column block's fragment stream
    const char* x;         // uniform: activations of the group
    int KS, K, M;          // fragments along K, K, rows of the group
    int n_chunks;          // chunks of U steps per wave
    int s0, sc;            // the steps of K this visit multiplies: s0 .. s0 + sc - 1 (all of them unless K is split)
    int spw;               // steps per wave: wave w owns the steps s0 + w * spw .. s0 + (w + 1) * spw - 1
    int rot;               // where in its range a wave starts (it wraps around): differs from tile to tile
};

// Activations of a step (two fragments = 128 bytes of K for MB x 16 rows) go through a per-wave LDS
// slot: direct-load instruction j covers rows 8j .. 8j+7 whole (8 x 128 bytes, eight cache lines),
// where loading MFMA operands straight from memory touches 16 half lines per instruction - the
// lines, not the bytes, are what the re-read of the activations costs next to the weight stream.
// Lane l of instruction j writes LDS chunk s = l%8 of row 8j + l/8 and fetches the global chunk
// c = s ^ ((row/2)%8); operand reads (16 rows x one chunk per quarter wave) then fall into 16
// different bank groups.
template <int DT, bool GATED, int MB, int NFR, int U>
__device__ __forceinline__ void skinny_setup(skinny_tile_state<NFR>& st, const epara_group_args& ga, int n0, int lane, int part, int nparts)
{
    constexpr int ESZ = DT == EPARA_BF16 ? 2 : 1;
    constexpr int EPC = 16 / ESZ, KF = 4 * EPC;
    const int K = ga.K, N = ga.N;
    const int KS = (K + KF - 1) / KF;
    const int NB = (N + 15) >> 4;
    st.K = K;
    st.KS = KS;
    const int steps = (KS + 1) >> 1;                             // two fragments per step
    st.s0 = 0;
    st.sc = steps;
    if (nparts > 1) {                                            // steps < 2^17, part < 8: the products fit 32 bits
        st.s0 = static_cast<int>(static_cast<uint32_t>(steps * part) / static_cast<uint32_t>(nparts));
        st.sc = static_cast<int>(static_cast<uint32_t>(steps * (part + 1)) / static_cast<uint32_t>(nparts)) - st.s0;
    }
    st.spw = max((st.sc + 3) >> 2, 1);
    st.n_chunks = (st.spw + U - 1) / U;
    // Tiles of one group that run at the same time would otherwise ask for the same activation lines (and
    // the same DRAM pages of their column blocks) at the same moment.  The start depends on the 128-column
    // span of the output only (every streaming class cuts a span into whole tiles), so a result is still a
    // function of the operands alone, whatever the class table and the grid.
    st.rot = static_cast<int>((static_cast<uint32_t>(n0 >> 7) * 2654435761u >> 12) % static_cast<uint32_t>(st.spw));
#pragma unroll
    for (int f = 0; f < NFR; ++f) {
        // gated: fragments 0 .. NFR/2-1 are gate blocks, the rest the same blocks of the up matrix
        const int rel = GATED ? (f % (NFR / 2)) : f;
        const int nb = min((n0 >> 4) + rel, NB - 1);             // a block past N only feeds unstored columns
        gcptr base = as_global<char>((GATED && f >= NFR / 2) ? ga.W2 : ga.W);
        st.w[f] = base + static_cast<size_t>(nb) * ((KS + 3) & ~3) * 1024;   // blocks are padded to a multiple of four stages
    }
    st.x = static_cast<const char*>(ga.X);
    st.M = ga.M;
}

// One ring slot: weight fragments ks = 2p and 2p+1 of NFR column blocks (the activations of the
// step sit in the wave's LDS slot of the same index).
template <int NFR>
struct skinny_slot { v4i w[2][NFR]; };

template <int DT, int MB, int NFR>
__device__ __forceinline__ void skinny_load(const skinny_tile_state<NFR>& st, int i, int wave, int lane, skinny_slot<NFR>& sl,
                                            char* xslot_generic)
{
    ldsptr xslot = (ldsptr)xslot_generic;
    constexpr int ESZ = DT == EPARA_BF16 ? 2 : 1;
    constexpr int EPC = 16 / ESZ, KF = 4 * EPC;
    int pi = min(i, st.spw - 1) + st.rot;                        // padding repeats the last step
    if (pi >= st.spw) pi -= st.spw;
    const int p = min(st.s0 + wave * st.spw + pi, ((st.KS + 1) >> 1) - 1);   // step: fragments 2p and 2p+1
    // activations first: loads complete in issue order, so once the weights of this slot are in
    // their registers the slot's LDS image is complete too
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(st.x), 0, -1, 0x00020000);
    // The lane's row offsets are worked out again at every step (a dozen integer instructions next to
    // kilobytes of loads): held in registers across the tile they are what gets spilled to scratch memory,
    // and a reload from there waits behind every weight load in flight.
    int l = lane;
    asm volatile("" : "+v"(l));
    const uint32_t row_bytes = static_cast<uint32_t>(st.K * ESZ);
    if ((2 * p + 2) * KF <= st.K) {                              // both fragments lie inside K
#pragma unroll
        for (int j = 0; j < 2 * MB; ++j) {
            const int row = 8 * j + (l >> 3);
            const int c = (l & 7) ^ ((row >> 1) & 7);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xrsrc, (__attribute__((address_space(3))) void*)(xslot + j * 1024), 16,
                                                     static_cast<int>(static_cast<uint32_t>(min(row, st.M - 1)) * row_bytes + c * 16), p * 128, 0, 0);
        }
    } else {
        // ragged or padding step: a fragment past the last one repeats the last, a chunk past K
        // falls back to chunk 0 of its fragment (the packed weights are zero there)
#pragma unroll
        for (int j = 0; j < 2 * MB; ++j) {
            const int row = 8 * j + (l >> 3);
            const int c = (l & 7) ^ ((row >> 1) & 7);
            const int ks = min(2 * p + (c >> 2), st.KS - 1);
            const int cc = (ks * KF + (c & 3) * EPC < st.K) ? (c & 3) : 0;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xrsrc, (__attribute__((address_space(3))) void*)(xslot + j * 1024), 16,
                                                     static_cast<int>(static_cast<uint32_t>(min(row, st.M - 1)) * row_bytes + ks * 64 + cc * 16), 0, 0, 0);
        }
    }
    const uint32_t lane16 = lane * 16;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int ks = min(2 * p + e, st.KS - 1);                // padding repeats the last fragment
#pragma unroll
        for (int f = 0; f < NFR; ++f) sl.w[e][f] = ld16(st.w[f] + static_cast<size_t>(ks) * 1024 + lane16);
    }
}

template <int DT, int MB, int NFR, int AFTER>
__device__ __forceinline__ void skinny_mma(const skinny_tile_state<NFR>& st, int i, int wave, int lane, const skinny_slot<NFR>& sl,
                                           char* xslot_generic, v4f (&acc)[NFR][MB])
{
    ldsptr xslot = (ldsptr)xslot_generic;
    // every load issued after this slot's belongs to one of the AFTER slots filled since
    wait_vmcnt<AFTER * (2 * NFR + 2 * MB)>();
    __builtin_amdgcn_sched_barrier(0);
    const int r = lane & 15, q = lane >> 4;
    v4i x[2][MB];
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int fm = 0; fm < MB; ++fm)
            x[e][fm] = *reinterpret_cast<lds_v4i>(xslot + (fm * 16 + r) * 128 + (((e * 4 + q) ^ ((r >> 1) & 7)) << 4));
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        int pi = i + st.rot;
        if (pi >= st.spw) pi -= st.spw;
        if (i < st.spw && wave * st.spw + pi < st.sc && 2 * (st.s0 + wave * st.spw + pi) + e < st.KS) {
#pragma unroll
            for (int f = 0; f < NFR; ++f)
#pragma unroll
                for (int fm = 0; fm < MB; ++fm) mma<DT>(acc[f][fm], sl.w[e][f], x[e][fm]);
        }
    }
}

// How a streaming tile's sums are laid out when they are reduced and finished.
template <bool GATED, int MB, int NFR>
struct skinny_shape {
    // red[wave][block of the pass][fm][lane]: at most 64 KiB, so the widest tile takes two passes
    static constexpr int PASSES = (NFR * MB * 4096 + RING_LDS_OFFSET - 1) / RING_LDS_OFFSET;
    static constexpr int NP = NFR / PASSES;                      // column blocks per pass
    static constexpr int QUADS = NFR * MB;                       // quads of 64 lanes in a tile's sums
    static constexpr int G2 = GATED ? 2 : 1;
    static constexpr int UNITS = GATED ? (NP / 2) * MB : NP * MB;   // per pass; a unit = one stored quad (gated: made of two)
    static constexpr int UPW = (UNITS + 3) / 4;                  // units per wave and pass
    static constexpr int BN = (GATED ? NFR / 2 : NFR) * 16;      // output columns of a tile
    static_assert(QUADS * 1024 <= SPLIT_STRIDE, "a tile's partial sums do not fit their workspace slot");
    // does the unit hold rows and columns of the group at all
    static __device__ __forceinline__ bool live(int pass, int unit, int M, int cols)
    {
        if (unit >= UNITS) return false;
        return (unit % MB) * 16 < M && (pass * (GATED ? NP / 2 : NP) + unit / MB) * 16 < cols;
    }
};

// Epilogue of one unit: the lane's quad of the sums (gated: gate and up) becomes four stored outputs.
template <class ActTag, bool GATED, int MB, int NFR, bool WT>
__device__ __forceinline__ void skinny_finish_unit(const epara_group_args& ga, int out_dtype, int n0, int cols, int pass, int unit,
                                                   const v4f& a, const v4f& b, int lane, bool vec_ok)
{
    typedef skinny_shape<GATED, MB, NFR> S;
    const int r = lane & 15, q = lane >> 4;
    const int hi = unit / MB, fm = unit % MB;
    if constexpr (GATED) {
        finish_gated<WT>(ga, out_dtype, a, b, 0, fm * 16 + r, ga.M, n0, (pass * (S::NP / 2) + hi) * 16 + 4 * q, cols, vec_ok);
    } else {
        finish_plain<ActTag::value, WT>(ga, out_dtype, a, ga.bias ? as_global<float>(ga.bias) + n0 : nullptr, 0,
                                        fm * 16 + r, ga.M, n0, (pass * S::NP + hi) * 16 + 4 * q, cols, vec_ok);
    }
}

// Reduces the four waves' partial sums of a tile in LDS (wave order) and finishes it.  When the tile's K is
// split over several visits (nparts > 1), the sums of this visit go to the workspace instead and the visit
// is noted in `pend`.  Returns whether the output tile was stored.
template <int DT, bool GATED, int MB, int NFR, bool WT>
__device__ __forceinline__ bool skinny_finish(const epara_group_args& ga, int out_dtype, int n0, int cols,
                                              v4f (&acc)[NFR][MB], int wave, int lane, char* lds,
                                              const split_ctx* sp, int entry, split_pending* pend)
{
    typedef skinny_shape<GATED, MB, NFR> S;
    constexpr int PASSES = S::PASSES, NP = S::NP, UNITS = S::UNITS, UPW = S::UPW, G2 = S::G2;
    // the scheduler splits neither the 16-row class, nor the phases of a chain (WT), nor fp8 tiles: no code for it there
    constexpr bool CAN_SPLIT = MB >= 2 && !WT && DT == EPARA_BF16;
    v4f* red = reinterpret_cast<v4f*>(lds);
    const bool vec_ok = (ga.N & 3) == 0;
    const int M = ga.M;
    auto dump = [&](int pass) {
        __syncthreads();                                         // the previous sums have been read
#pragma unroll
        for (int fi = 0; fi < NP; ++fi) {
            // gated: a pass holds NP/2 gate blocks and the matching up blocks
            const int f = GATED ? (fi < NP / 2 ? pass * (NP / 2) + fi : NFR / 2 + pass * (NP / 2) + fi - NP / 2) : pass * NP + fi;
#pragma unroll
            for (int fm = 0; fm < MB; ++fm) red[((wave * NP + fi) * MB + fm) * 64 + lane] = acc[f][fm];
        }
        __syncthreads();
    };
    auto sum = [&](int unit, v4f& a, v4f& b) {
        const int hi = unit / MB, fm = unit % MB;                // plain: the block; gated: the gate / up block pair
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            a += red[((w * NP + hi) * MB + fm) * 64 + lane];
            if constexpr (GATED) b += red[((w * NP + NP / 2 + hi) * MB + fm) * 64 + lane];
        }
    };
    if constexpr (CAN_SPLIT) {
        const int nparts = order_parts(entry);
        if (nparts > 1) {
            // An order that asks for parts without a workspace, or for more parts than a slot holds, is not one
            // the library's planner writes (the host cannot see the device copy of the order): the visit is
            // dropped rather than let it write through a null or past its slot.
            // the tile's slot = the group's first slot + its column tile; quad index = (pass, unit[, gate / up])
            const int slot = ga.reserved + n0 / S::BN;
            if (sp->ws == nullptr || nparts > SPLIT_MAX_PARTS || ga.reserved < 0 || slot >= sp->n_split) return false;
            char* mine = split_partials(*sp) + (static_cast<size_t>(slot) * SPLIT_MAX_PARTS + order_part(entry)) * SPLIT_STRIDE + lane * 16;
#pragma unroll
            for (int pass = 0; pass < PASSES; ++pass) {
                dump(pass);
#pragma unroll
                for (int k = 0; k < UPW; ++k) {
                    const int unit = wave + 4 * k;
                    if (!S::live(pass, unit, M, cols)) continue;
                    v4f a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
                    sum(unit, a, b);
                    char* at = mine + static_cast<size_t>((pass * UNITS + unit) * G2) * 1024;
                    split_put(at, a);
                    if constexpr (GATED) split_put(at + 1024, b);
                }
            }
            if (lane == pend->count) { pend->slots = slot | ((nparts - 1) << 28); pend->entries = entry; }
            ++pend->count;
            return false;
        }
    }
    auto run = [&](auto tag) {
#pragma unroll
        for (int pass = 0; pass < PASSES; ++pass) {
            dump(pass);
            for (int unit = wave; unit < UNITS; unit += 4) {
                if (!S::live(pass, unit, M, cols)) continue;
                v4f a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
                sum(unit, a, b);
                skinny_finish_unit<decltype(tag), GATED, MB, NFR, WT>(ga, out_dtype, n0, cols, pass, unit, a, b, lane, vec_ok);
            }
        }
    };
    if constexpr (GATED) run(act_tag<EPARA_ACT_SILU>{});
    else                 with_act(ga.act, run);
    return true;
}

// The visit that arrived last at a split tile: the parts come back from the workspace (straight into the LDS,
// every wave those of the units it finishes, so no barrier), are added in index order, whoever wrote them last,
// and the tile is finished.
template <int DT, bool GATED, int MB, int NFR>
__device__ __forceinline__ void split_finish(const epara_group_args& ga, int out_dtype, int n0, int cols, int slot, int nparts,
                                             int wave, int lane, char* lds, const split_ctx* sp)
{
    typedef skinny_shape<GATED, MB, NFR> S;
    constexpr int PASSES = S::PASSES, NP = S::NP, UNITS = S::UNITS, UPW = S::UPW, G2 = S::G2;
    const v4f* red = reinterpret_cast<const v4f*>(lds);
    const bool vec_ok = (ga.N & 3) == 0;
    const int M = ga.M;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        split_partials(*sp) + static_cast<size_t>(slot) * SPLIT_MAX_PARTS * SPLIT_STRIDE, 0, -1, 0x00020000);
    auto run = [&](auto tag) {
#pragma unroll 1
        for (int pass = 0; pass < PASSES; ++pass) {
#pragma unroll
            for (int k = 0; k < UPW; ++k) {
                const int unit = wave + 4 * k;
                if (!S::live(pass, unit, M, cols)) continue;
                for (int pt = 0; pt < nparts; ++pt)
#pragma unroll
                    for (int h = 0; h < G2; ++h)
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(
                            rsrc, (__attribute__((address_space(3))) void*)((ldsptr)lds + (((pt * UNITS + unit) * G2 + h) << 10)), 16,
                            lane * 16, pt * SPLIT_STRIDE + (((pass * UNITS + unit) * G2 + h) << 10), 0, 16);   // 16: device scope (sc1)
            }
            wait_vmcnt<0>();
            asm volatile("" ::: "memory");
#pragma unroll
            for (int k = 0; k < UPW; ++k) {
                const int unit = wave + 4 * k;
                if (!S::live(pass, unit, M, cols)) continue;
                v4f a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
                for (int pt = 0; pt < nparts; ++pt) {
                    a += red[((pt * UNITS + unit) * G2) * 64 + lane];
                    if constexpr (GATED) b += red[((pt * UNITS + unit) * G2 + 1) * 64 + lane];
                }
                skinny_finish_unit<decltype(tag), GATED, MB, NFR, false>(ga, out_dtype, n0, cols, pass, unit, a, b, lane, vec_ok);
            }
            wait_lgkmcnt0();                                     // the sums are in registers before the next pass lands on them
        }
    };
    if constexpr (GATED) run(act_tag<EPARA_ACT_SILU>{});
    else                 with_act(ga.act, run);
}

// The last chunk of a run: slot I has U - 1 - I slots issued after it and nothing is refilled.
template <int DT, int MB, int NFR, int U, int I>
__device__ __forceinline__ void skinny_drain(const skinny_tile_state<NFR>& st, int c, int wave, int lane, const skinny_slot<NFR> (&ring)[U],
                                             char* xring, v4f (&acc)[NFR][MB])
{
    if constexpr (I < U) {
        skinny_mma<DT, MB, NFR, U - 1 - I>(st, c * U + I, wave, lane, ring[I], xring + I * (MB * 2048), acc);
        __builtin_amdgcn_sched_barrier(0);
        skinny_drain<DT, MB, NFR, U, I + 1>(st, c, wave, lane, ring, xring, acc);
    }
}

// What a run has already read about the slot that follows it in the workgroup's list: the next run starts
// without the three dependent loads (order -> tile -> group arguments), which cost microseconds each while
// the whole chip streams weights.
struct run_next {
    bool known;            // entry, tl and ga below are those of the slot the run returned
    int entry;
    epara_tile tl;
    epara_group_args ga;
};

// Processes slot `slot` (its order entry and tile and, if first_ga_known, its group arguments already read)
// and every following slot of this workgroup that holds a tile of the same streaming class.  Returns the
// first slot it did not process (n_slots at the end of the list; a list has no holes) and what it knows of it.
template <int DT, bool GATED, bool CHAIN, int CLS, int MB, int NFR, int U>
__device__ __forceinline__ long skinny_run(const epara_group_args* __restrict__ args, const epara_tile* __restrict__ tiles,
                                           const int32_t* __restrict__ order, long slot, int entry, const epara_tile& first_tile,
                                           const epara_group_args& first_ga, bool first_ga_known, long n_slots, long stride,
                                           int out_dtype, char* lds, chain_ctx* chain, const split_ctx* sp, split_pending* pend,
                                           run_next& following)
{
    // The thread index passes through an empty asm: what a run derives from it (lane offsets, swizzles) is then
    // computed here, per run, instead of once for the whole kernel, where such values stay alive across the
    // other tile classes' code and end up in scratch memory.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    epara_tile tl = first_tile;                                  // entry: the tile, and which part of its K (see order_tile)
    epara_group_args ga;
    if (first_ga_known) ga = first_ga;
    else                ga = args[tl.group];
    skinny_tile_state<NFR> cur, nxt;
    skinny_setup<DT, GATED, MB, NFR, U>(cur, ga, tl.n0, lane, order_part(entry), order_parts(entry));
    skinny_slot<NFR> ring[U];
    constexpr int XSLOT_BYTES = MB * 2048;
    char* xring = lds + RING_LDS_OFFSET + wave * (U * XSLOT_BYTES);
    static_assert(RING_LDS_OFFSET + 4 * U * XSLOT_BYTES <= LDS_BYTES, "activation rings do not fit");
    // The rings overlay whatever used this part of the LDS before (a panel tile's epilogue, the
    // rings of another streaming class: a run ends with every slot consumed, nothing in flight).
    __syncthreads();
#pragma unroll
    for (int u = 0; u < U; ++u) skinny_load<DT, MB, NFR>(cur, u, wave, lane, ring[u], xring + u * XSLOT_BYTES);
    __builtin_amdgcn_sched_barrier(0);

    for (;;) {
        // What follows this tile in the workgroup's list (a list has no holes, so an idle slot ends
        // it) is found by three dependent scalar loads: order -> tile -> group arguments.  Each
        // link is issued after one chunk of the tile and read after the next, so that its latency
        // passes while the wave waits for weights anyway instead of stopping the stream.
        int t_next = -1, stage = 0;                              // t_next: the order entry that follows
        bool have_next = false;
        epara_tile tl_next = tl;
        epara_group_args ga_next = ga;
        auto advance = [&]() {
            if (stage == 0)      { const long s1 = slot + stride; t_next = s1 < n_slots ? order[s1] : -1; }
            else if (stage == 1) { if (t_next >= 0) tl_next = tiles[order_tile(t_next)]; }
            else {
                have_next = t_next >= 0 && tl_next.cls == CLS;
                // the run ends while the list of uncounted visits still has room for one more
                if constexpr (!CHAIN && MB >= 2 && DT == EPARA_BF16) have_next = have_next && pend->count < 63;
                // in a chain the run ends before a tile that may have to wait for its input
                if constexpr (CHAIN) have_next = have_next && (tl_next.group == tl.group || !chain_must_wait(*chain, tl_next.group));
                if (t_next >= 0) ga_next = args[tl_next.group]; // also when another kind of run takes the slot: it starts from these
            }
            ++stage;
        };
        v4f acc[NFR][MB];
#pragma unroll
        for (int f = 0; f < NFR; ++f)
#pragma unroll
            for (int fm = 0; fm < MB; ++fm) acc[f][fm] = v4f{0.f, 0.f, 0.f, 0.f};
        for (int c = 0; c + 1 < cur.n_chunks; ++c) {             // refill from this tile
#pragma unroll
            for (int u = 0; u < U; ++u) {
                skinny_mma<DT, MB, NFR, U - 1>(cur, c * U + u, wave, lane, ring[u], xring + u * XSLOT_BYTES, acc);
                __builtin_amdgcn_sched_barrier(0);
                skinny_load<DT, MB, NFR>(cur, (c + 1) * U + u, wave, lane, ring[u], xring + u * XSLOT_BYTES);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (stage < 3) advance();
            __builtin_amdgcn_sched_barrier(0);
        }
        while (stage < 3) advance();                             // short tiles: the rest of the chain at once
        const long slot_next = have_next ? slot + stride : -1L;
        const int c_last = cur.n_chunks - 1;
        if (have_next) {                                         // last chunk: refill from the next tile
            skinny_setup<DT, GATED, MB, NFR, U>(nxt, ga_next, tl_next.n0, lane, order_part(t_next), order_parts(t_next));
#pragma unroll
            for (int u = 0; u < U; ++u) {
                skinny_mma<DT, MB, NFR, U - 1>(cur, c_last * U + u, wave, lane, ring[u], xring + u * XSLOT_BYTES, acc);
                __builtin_amdgcn_sched_barrier(0);
                skinny_load<DT, MB, NFR>(nxt, u, wave, lane, ring[u], xring + u * XSLOT_BYTES);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {                                                 // nothing follows: the ring drains
            skinny_drain<DT, MB, NFR, U, 0>(cur, c_last, wave, lane, ring, xring, acc);
        }
        const bool stored = skinny_finish<DT, GATED, MB, NFR, CHAIN>(ga, out_dtype, tl.n0, tl.cols, acc, wave, lane, lds, sp, entry, pend);
        if constexpr (CHAIN) { if (stored) chain_done(*chain, tl.group); }
        if (slot_next < 0) {                                     // the run ends here: hand over what is known of the next slot
            following.known = t_next >= 0;
            following.entry = t_next;
            following.tl = tl_next;
            following.ga = ga_next;
            slot = t_next >= 0 ? slot + stride : n_slots;
            break;
        }
        slot = slot_next;
        entry = t_next;
        tl = tl_next;
        ga = ga_next;
        cur = nxt;
    }
    return slot;
}

}  // namespace

#endif
