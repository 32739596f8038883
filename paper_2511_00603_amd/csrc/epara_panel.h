// Panel tiles of libepara: big batches on the matrix cores (gfx950).
//
// A panel tile is 256 rows x 256 columns of one group (gated groups: 256 rows x 128 hidden columns,
// i.e. 128 gate + 128 up weight columns).  The four waves of the workgroup (one per SIMD, the whole
// register file each) split the tile by COLUMNS: wave w owns all 256 rows of columns 64 w .. 64 w + 63
// (gated: hidden columns 32 w .. 32 w + 31 = one 32-column fragment of the gate matrix and the same
// columns of the up matrix), i.e. 2 x 8 accumulator fragments of 32 x 32 = 256 registers.
//
//   weights      belong to one wave only, so they never touch the LDS: a wave-wide 16-byte load of the
//                packed layout is already an MFMA operand (plain buffer loads into a register ring of
//                four K stages, refilled four stages ahead, each register right after its last use);
//   activations  are shared by all four waves: direct global->LDS loads (no staging registers) into a
//                ring of four buffers of 256 rows x 128 bytes (a "pair" of two 64-byte K stages; whole
//                cache lines), XOR-swizzled so that fragment reads are free of bank conflicts.  Wave w
//                fetches rows 64 w .. 64 w + 63 of every pair; one workgroup barrier per pair.
//
// All panel tiles that follow each other in a workgroup's list form ONE software pipeline: the
// loaders (activations four pairs ahead, weights four stages ahead) walk the list on their own and
// cross tile boundaries, so the operands of the next tile are in flight while this tile's epilogue
// runs, and its first MFMA issues right after.  The pipeline issues the same number of loads in
// every step from its cold start to its end (past the end of the run: re-loads of the last data into
// places nobody reads), which is what makes "my part of pair p has landed" a constant bound on the
// number of loads still in flight: loads complete in issue order.
//
// K is walked two pairs (four 64-byte stages) at a time, which keeps every register index of the weight
// ring a compile-time constant; a tile whose K is not a multiple of four stages multiplies up to
// three stages of zeros: the packed weights are padded to a multiple of four stages
// (epara_pack_weights).  Activation chunks past K are fetched from chunk 0 of the row instead (finite
// values against zero weights).  Rows past the batch and column blocks past N are clamped to the last valid one (they
// only feed outputs that are never stored).
//
// Epilogue.  The 256 accumulators of a lane sit in the AGPR half of the register file.  Per 32-row
// fragment row the wave parks them in its own 8 KiB of LDS (outside the operand ring, which already
// holds the next tile) and reads them back transposed, one quad (4 consecutive columns of one row) per
// lane, so that a store instruction writes whole row pieces of 128 bytes (gated: 64).
#ifndef EPARA_PANEL_H
#define EPARA_PANEL_H

#include "epara_device.h"

namespace {

constexpr int XPAIR_BYTES = 32768;                       // 256 rows x 128 B
constexpr int XRING = 4;
constexpr int STASH_LDS_OFFSET = XRING * XPAIR_BYTES;    // 8 KiB per wave
static_assert(STASH_LDS_OFFSET + 4 * 8192 <= LDS_BYTES, "operand ring and stash do not fit");
// Loads issued between the last activation load of pair p + 1 and the barrier that ends pair p: two
// pairs' worth (8 activation + 8 weight loads per pair).
constexpr int PANEL_LOADS_PER_PAIR = 16;

struct panel_walker { long slot; int t; epara_tile tl; int nsplit; };   // nsplit: visits to parts of tiles so far in the run

template <int DT, bool GATED, bool WT, bool CHAIN>
__device__ __forceinline__ long panel_run(const epara_group_args* __restrict__ args, const epara_tile* __restrict__ tiles,
                                          const int32_t* __restrict__ order, long slot0, long n_slots, long stride,
                                          int out_dtype, char* lds, chain_ctx* chain, const split_ctx* sp = nullptr,
                                          split_pending* pend = nullptr)
{
    // Tiles of the launch's last round may be visited in parts of K (plain bf16 groups of a single launch only): an
    // entry of the order then names the part, the three walkers cover that part's units of four stages only,
    // and the visit leaves its raw sums in the workspace instead of running the epilogue.
    constexpr bool CAN_SPLIT = !GATED && !CHAIN && !WT && DT == EPARA_BF16;
    constexpr int ESZ = DT == EPARA_BF16 ? 2 : 1;
    constexpr int EPC = 16 / ESZ;   // elements per 16-byte chunk
    constexpr int KF = 4 * EPC;     // K elements per stage
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));                               // what is derived from it is computed per run (see skinny_run)
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r32 = lane & 31, h = lane >> 5;
    ldsptr l3 = (ldsptr)lds;
    // units (of two pairs = four stages) of K that the visit `entry` of a tile with KD pairs covers: [u0, u1)
    auto unit_range = [&](int entry, int KD, int& u0, int& u1) {
        u0 = 0; u1 = KD >> 1;
        if constexpr (CAN_SPLIT) {
            const int parts = order_parts(entry);
            if (parts > 1) {
                const uint32_t U = static_cast<uint32_t>(KD >> 1), part = static_cast<uint32_t>(order_part(entry));
                u0 = static_cast<int>(U * part / static_cast<uint32_t>(parts));
                u1 = static_cast<int>(U * (part + 1) / static_cast<uint32_t>(parts));
            }
        }
    };

    // ---- walking the workgroup's list.  Three consumers (activation loader, weight loader, multiply +
    // epilogue) each hold their own position; w_next moves one to the following tile of the run or
    // marks it ended (t < 0; sticky).  In a chain a run ends before a group that waits for its input.
    const int split_room = CAN_SPLIT ? 63 - pend->count : 0;     // the caller leaves room for at least one
    auto w_next = [&](panel_walker& w) {
        if (w.t < 0) return;
        const int group = w.tl.group;
        w.slot += stride;
        int t = w.slot < n_slots ? order[w.slot] : -1;
        if (t >= 0) {
            const epara_tile tl = tiles[order_tile(t)];          // (an entry of a streaming tile may name a part of K)
            bool ok = tl.cls >= N_STREAM_CLASSES;
            if constexpr (CHAIN) {
                if (ok && chain->waits != nullptr && tl.group != group) {
                    const epara_chain_wait cw = chain->waits[tl.group];
                    ok = !(cw.counter >= 0 && cw.need > 0);
                }
            }
            if constexpr (CAN_SPLIT) {                           // the run ends while the list of uncounted visits has room
                if (ok && order_parts(t) > 1) ok = w.nsplit++ < split_room;
            }
            if (ok) w.tl = tl; else t = -1;
        }
        w.t = t;
    };
    const panel_walker first = {slot0, order[slot0], tiles[order_tile(order[slot0])], (CAN_SPLIT && order_parts(order[slot0]) > 1) ? 1 : 0};

    // ---- activation loader: wave w fetches rows 64 w + 8 j + lane / 8 with instruction j = 0..7 of a pair;
    // lane l writes LDS slot l % 8 of its row and fetches the global chunk that belongs there.
    panel_walker xw = first;
    __amdgpu_buffer_rsrc_t xrsrc;
    uint32_t x_off[8];                                           // byte offset of my row + my chunk
    int x_pair = 0, x_KD = 2, x_K = 0, x_ring = XRING - 1;
    const int x_chunk[2] = {(lane & 7) ^ ((lane >> 4) & 7), (lane & 7) ^ ((4 + (lane >> 4)) & 7)};   // = slot ^ ((row/2) % 8), j even / odd
    auto x_enter = [&]() {
        const epara_group_args& ga = args[xw.tl.group];
        const int K = ga.K;
        xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(static_cast<const char*>(ga.X)) +
                                                  static_cast<size_t>(xw.tl.m0) * K * ESZ, 0, -1, 0x00020000);
#pragma unroll
        for (int j = 0; j < 8; ++j)
            x_off[j] = static_cast<uint32_t>(min(64 * wave + 8 * j + (lane >> 3), xw.tl.rows - 1)) * static_cast<uint32_t>(K * ESZ) +
                       static_cast<uint32_t>(x_chunk[j & 1] * 16);
        int u0, u1;
        unit_range(xw.t, ((K + KF - 1) / KF + 3) >> 2 << 1, u0, u1);   // pairs: an even number
        x_pair = 2 * u0;                                         // first pair of the visit
        x_KD = 2 * u1;                                           // one past its last
        x_K = K;
    };
    auto x_issue = [&](int j) {
        uint32_t off = x_off[j];
        int so = x_pair * 128;
        const int left = x_K - x_pair * 2 * KF;                 // elements of K from this pair on
        if (left < 2 * KF) {                                     // last pair(s) of a ragged K: chunks past K come from chunk 0
            const int c = x_chunk[j & 1];
            if (c * EPC >= left) off -= static_cast<uint32_t>(c * 16);
            if (left <= 0) so = 0;
        }
        __builtin_amdgcn_raw_ptr_buffer_load_lds(xrsrc, (__attribute__((address_space(3))) void*)(l3 + x_ring * XPAIR_BYTES + (8 * wave + j) * 1024),
                                                 16, off, so, 0, 0);
    };
    auto x_advance = [&]() {                                     // on to the next pair of the run, into the ring slot just freed
        x_ring = (x_ring + 1) & (XRING - 1);
        if (xw.t < 0) return;                                    // past the end: the same pair again
        if (++x_pair == x_KD) {
            w_next(xw);
            if (xw.t >= 0) x_enter(); else x_pair = x_KD - 1;
        }
    };

    // ---- weight loader: fragment fn of wave w is two packed column blocks side by side; lane (r32, h) takes
    // chunk 2 s2 + h of column r32 % 16 of block r32 / 16 for step s2 of a stage.
    panel_walker ww = first;
    __amdgpu_buffer_rsrc_t wrsrc[2];
    uint32_t w_off[2];
    int w_stage = 0, w_KSP = 4;
    auto w_enter = [&]() {
        const epara_group_args& ga = args[ww.tl.group];
        const int K = ga.K, N = ga.N;
        const int KSP = (((K + KF - 1) / KF) + 3) & ~3;
        const int NB = (N + 15) >> 4;
        const int nb0 = min((ww.tl.n0 >> 4) + (GATED ? 2 : 4) * wave, NB - 1);
#pragma unroll
        for (int fn = 0; fn < 2; ++fn) {
            const int rel = min((GATED ? 0 : 2 * fn) + (r32 >> 4), NB - 1 - nb0);
            w_off[fn] = static_cast<uint32_t>(rel) * static_cast<uint32_t>(KSP) * 1024u + static_cast<uint32_t>((h * 16 + (r32 & 15)) * 16);
            const void* base = (GATED && fn == 1) ? ga.W2 : ga.W;
            wrsrc[fn] = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(static_cast<const char*>(base)) +
                                                          static_cast<size_t>(nb0) * KSP * 1024, 0, -1, 0x00020000);
        }
        int u0, u1;
        unit_range(ww.t, KSP >> 1, u0, u1);
        w_stage = 4 * u0;                                        // first stage of the visit
        w_KSP = 4 * u1;                                          // one past its last
    };
    auto w_issue = [&](int fn, int s2) -> v4i {
        return __builtin_amdgcn_raw_buffer_load_b128(wrsrc[fn], w_off[fn] + s2 * 512, w_stage * 1024, 0);
    };
    auto w_advance = [&]() {
        if (ww.t < 0) return;
        if (++w_stage == w_KSP) {
            w_next(ww);
            if (ww.t >= 0) w_enter(); else w_stage = w_KSP - 1;
        }
    };

    // ---- fragment reads: rows fm * 32 + r32 of the pair in ring slot `ring`, chunk c = 0..7 of the pair at
    // position c ^ ((row / 2) % 8); (row / 2) % 8 does not depend on fm.
    const int sw = (r32 >> 1) & 7;
    uint32_t xf_off[4];                                          // chunk pairs (2 i + h), i = 0..3
#pragma unroll
    for (int i = 0; i < 4; ++i) xf_off[i] = static_cast<uint32_t>(r32 * 128 + (((2 * i + h) ^ sw) << 4));
    auto read_frag = [&](int ring, int i, int fm) -> v4i {
        return *reinterpret_cast<lds_v4i>(l3 + ring * XPAIR_BYTES + xf_off[i] + fm * 4096);
    };

    // ---- cold start: nothing of an earlier tile is in flight or being read; fill the ring and the weight
    // registers (four pairs, four stages) and wait for all of it once.
    v4i wreg[4][2][2];                                           // [stage % 4][fn][s2]
    v4i xf[2][8];
    wait_vmcnt<0>();
    __syncthreads();
    x_enter();
    w_enter();
#pragma unroll
    for (int p = 0; p < XRING; ++p) {
        if (p > 0) x_advance(); else x_ring = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) x_issue(j);
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
#pragma unroll
        for (int fn = 0; fn < 2; ++fn)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                // the last registers of stage 3 are left to the first step, which refills "the registers
                // the step before used last" like every other step
                const bool later = s == 3 && fn == 1 && (DT != EPARA_BF16 || s2 == 1);
                if (!later) wreg[s][fn][s2] = w_issue(fn, s2);
            }
        if (s < 3) w_advance();
    }
    wait_vmcnt<0>();
    __syncthreads();
    int rd_ring = 0;
    if constexpr (DT == EPARA_BF16) {
#pragma unroll
        for (int fm = 0; fm < 8; ++fm) xf[0][fm] = read_frag(0, 0, fm);
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) xf[0][i] = read_frag(0, i >> 2, i & 3);
    }

    // ---- one step = a quarter of a pair: bf16: stage S = T / 2, K half s2 = T % 2, 16 MFMAs 32x32x16 over
    // 2 x 8 fragments; fp8: stage S, row half T % 2, 8 MFMAs 32x32x64 over 2 x 4 fragments.  During a
    // step the fragments of the next step are read into the other register set, weight registers are
    // refilled (stage + 4) right after their last use -- those of fragment 1 at the start of the
    // following step -- and two activation loads of the pair that goes into the ring slot freed at the
    // last barrier are issued.  A wave issues in order and a memory instruction can take most of an
    // MFMA's run time to leave the wave (the four waves share one address unit), so there is at most one
    // of them between two MFMAs (fp8, whose MFMAs run twice as long: two), pinned by the scheduling
    // barriers: two in a row leave the matrix core idle.  Every step issues exactly four loads.
    // PH = parity of the pair: which half of the weight ring.
    v16f acc[2][8];
    auto step = [&](auto ph_tag, auto t_tag) {
        constexpr int PH = decltype(ph_tag)::value, T = decltype(t_tag)::value;
        constexpr int S = T >> 1, slot = 2 * PH + S, set = T & 1, NT1 = (T + 1) & 3;
        constexpr int pslot = T == 0 ? 2 * (PH ^ 1) + 1 : 2 * PH + ((T - 1) >> 1);   // weight ring slot of the step before
        if constexpr (T == 3) {
            wait_lgkmcnt0();                                     // every fragment of this pair is in registers
            wait_vmcnt<2 * PANEL_LOADS_PER_PAIR>();              // my part of the next pair has landed
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            x_advance();                                         // the slot of this pair is free
        }
        const int nring = T == 3 ? ((rd_ring + 1) & (XRING - 1)) : rd_ring;
        if constexpr (DT == EPARA_BF16) {
            constexpr int s2 = T & 1, ps2 = s2 ^ 1;
#pragma unroll
            for (int m = 0; m < 16; ++m) {
                constexpr int rd[16] = {-1, 0, 1, 2, -1, 3, 4, 5, -1, 6, 7, -1, -1, -1, -1, -1};   // fragment read after MFMA m
                const int fn = m >> 3, fm = m & 7;
                mma32<DT>(acc[fn][fm], wreg[slot][fn][s2], xf[set][fm]);
                if (m == 0) {
                    wreg[pslot][1][ps2] = w_issue(1, ps2);
                    if (ps2 == 1) w_advance();
                }
                if (m == 4) x_issue(2 * NT1);
                if (m == 8) wreg[slot][0][s2] = w_issue(0, s2);
                if (m == 12) x_issue(2 * NT1 + 1);
                if (rd[m] >= 0) xf[set ^ 1][rd[m]] = read_frag(nring, NT1, rd[m]);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            typedef int v8i __attribute__((ext_vector_type(8)));
            constexpr int half = T & 1;                          // fragments fm = 4 half .. 4 half + 3; xf[set][e * 4 + fmi] = chunk (e ? 2 + h : h)
            constexpr int NS = NT1 >> 1, nhalf = NT1 & 1;
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                constexpr int rd[2][8] = {{-1, 0, -1, 1, 2, 3, -1, -1}, {0, 1, -1, -1, 2, 3, -1, -1}};   // [half][m]: fragment (both chunks) read after MFMA m
                const int fn = m >> 2, fmi = m & 3;
                const v8i a8 = __builtin_shufflevector(wreg[slot][fn][0], wreg[slot][fn][1], 0, 1, 2, 3, 4, 5, 6, 7);
                const v8i b8 = __builtin_shufflevector(xf[set][fmi], xf[set][4 + fmi], 0, 1, 2, 3, 4, 5, 6, 7);
                acc[fn][4 * half + fmi] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, acc[fn][4 * half + fmi], 0, 0, 0, 0, 0, 0);
                if (half == 0 && m == 0) {                       // the step before was the second half of a stage: its fragment 1 is free
                    wreg[pslot][1][0] = w_issue(1, 0);
                    wreg[pslot][1][1] = w_issue(1, 1);
                    w_advance();
                }
                if (half == 1 && m == 3) {
                    wreg[slot][0][0] = w_issue(0, 0);
                    wreg[slot][0][1] = w_issue(0, 1);
                }
                if (m == 2) x_issue(2 * NT1);
                if (m == 6) x_issue(2 * NT1 + 1);
                if (rd[half][m] >= 0) {
                    xf[set ^ 1][rd[half][m]] = read_frag(nring, 2 * NS, 4 * nhalf + rd[half][m]);
                    xf[set ^ 1][4 + rd[half][m]] = read_frag(nring, 2 * NS + 1, 4 * nhalf + rd[half][m]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if constexpr (T == 3) rd_ring = nring;
    };
    auto pair = [&](auto ph_tag) {
        step(ph_tag, act_tag<0>{});
        step(ph_tag, act_tag<1>{});
        step(ph_tag, act_tag<2>{});
        step(ph_tag, act_tag<3>{});
    };

    // ---- the tiles of the run
    panel_walker cw = first;
    v4f* stash = reinterpret_cast<v4f*>(lds + STASH_LDS_OFFSET) + wave * 512;
    for (;;) {
        const epara_group_args ga = args[cw.tl.group];
        const int m0 = cw.tl.m0, n0 = cw.tl.n0, rows = cw.tl.rows, cols = cw.tl.cols, N = ga.N;
        int u0, u1;
        unit_range(cw.t, ((ga.K + KF - 1) / KF + 3) >> 2 << 1, u0, u1);
        const int KD = 2 * (u1 - u0);                            // pairs of this visit, an even number
        // epilogue layout: QPR lanes share a row of this wave's part of the tile (64 columns; gated: 32), 4 columns each
        constexpr int QPR = GATED ? 8 : 16, RPI = 64 / QPR, WCOLS = 4 * QPR;
        const int q = lane % QPR, rr = lane / QPR;
        const int nl = wave * WCOLS + 4 * q;                     // first of this lane's four columns, relative to n0
        const bool vec_ok = (N & 3) == 0;
        v4f b4 = {0.f, 0.f, 0.f, 0.f};                           // fetched now so that nobody waits for it later
        if (!GATED && ga.bias) {
            const EPARA_GLOBAL float* bp = as_global<float>(ga.bias) + n0 + nl;
            if (nl + 3 < cols) b4 = *reinterpret_cast<const EPARA_GLOBAL v4f*>(bp);
            else {
#pragma unroll
                for (int i = 0; i < 4; ++i) if (nl + i < cols) b4[i] = bp[i];
            }
        }
#pragma unroll
        for (int fn = 0; fn < 2; ++fn)
#pragma unroll
            for (int fm = 0; fm < 8; ++fm)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[fn][fm][v] = 0.f;
        for (int c = 0; c < KD; c += 2) {
            pair(act_tag<0>{});
            pair(act_tag<1>{});
        }

        // ---- epilogue (the loads of the following tile stay in flight; only this wave's stash is used).
        // One wave per SIMD cannot overlap this with anybody's MFMAs, so what counts is the number of
        // instructions: a whole tile (the common case) runs fully unrolled with constant LDS offsets, no
        // bounds checks and one uniform pointer; ragged tiles run a compact loop with the checks.
        if constexpr (CAN_SPLIT) {
            const int nparts = order_parts(cw.t);
            if (nparts > 1) {
                // this visit's raw sums, row-major 256 x 256 fp32, written through to memory; counted when the
                // workgroup's list ends (an order that names parts the launch has no room for is dropped)
                const int pslot = order_tile(cw.t) - sp->first_panel;
                if (sp->ws != nullptr && nparts <= SPLIT_MAX_PARTS && pslot >= 0 && pslot < sp->n_panel) {
                    char* mine = panel_partials(*sp) + (static_cast<size_t>(pslot) * SPLIT_MAX_PARTS + order_part(cw.t)) * PANEL_SPLIT_STRIDE +
                                 static_cast<size_t>(wave * 64 + 4 * (lane & 15)) * 4;
                    auto raw = [&](auto fm_tag) {
                        constexpr int fm = decltype(fm_tag)::value;
                        if (fm * 32 >= rows) return;
                        // the park of the epilogue below (it is defined there): fragment row fm into the stash
#pragma unroll
                        for (int fn = 0; fn < 2; ++fn)
#pragma unroll
                            for (int g = 0; g < 4; ++g)
                                stash[r32 * 16 + ((fn * 8 + 2 * g + h) ^ (r32 & 15))] =
                                    v4f{acc[fn][fm][4 * g], acc[fn][fm][4 * g + 1], acc[fn][fm][4 * g + 2], acc[fn][fm][4 * g + 3]};
#pragma unroll
                        for (int it = 0; it < 8; ++it) {         // 16 lanes share a row: 4 rows per instruction
                            const int row = it * 4 + (lane >> 4);
                            split_put16(mine + static_cast<size_t>(fm * 32 + row) * 1024, stash[row * 16 + ((lane & 15) ^ (row & 15))]);
                        }
                    };
                    raw(act_tag<0>{}); raw(act_tag<1>{}); raw(act_tag<2>{}); raw(act_tag<3>{});
                    raw(act_tag<4>{}); raw(act_tag<5>{}); raw(act_tag<6>{}); raw(act_tag<7>{});
                    if (lane == pend->count) { pend->slots = (sp->n_split + pslot) | ((nparts - 1) << 28); pend->entries = cw.t; }
                    ++pend->count;
                }
                w_next(cw);
                if (cw.t < 0) break;
                continue;
            }
        }
        const float sg = ga.scale, s2g = ga.scale2 * ga.out_inv_scale, inv = ga.out_inv_scale;
        // Fragment row fm of this wave into its stash: 32 rows x 16 quads (fragment fn = 0 / 1: quads 0..7 / 8..15;
        // gated: gate / up), quad c of row r at position c ^ (r % 16): the writes (16 rows of one quad per
        // quarter wave) and the reads (the quads of a row side by side) both touch 16 different bank groups.
        auto park = [&](auto fm_tag) {
            constexpr int fm = decltype(fm_tag)::value;
#pragma unroll
            for (int fn = 0; fn < 2; ++fn)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    stash[r32 * 16 + ((fn * 8 + 2 * g + h) ^ (r32 & 15))] =
                        v4f{acc[fn][fm][4 * g], acc[fn][fm][4 * g + 1], acc[fn][fm][4 * g + 2], acc[fn][fm][4 * g + 3]};
        };
        // The four outputs of this lane in row `row` of the parked fragment row: plain groups act(s a + b),
        // gated groups SiLU(s gate) * (s2 up) from the gate quad and the up quad of the same hidden columns.
        auto finish = [&](auto act, int row, float (&v)[4]) {
            constexpr int ACT = decltype(act)::value;
            if constexpr (GATED) {
                const v4f gq = stash[row * 16 + (q ^ (row & 15))], uq = stash[row * 16 + ((8 + q) ^ (row & 15))];
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = act_fast<EPARA_ACT_SILU>(sg * gq[i]) * (s2g * uq[i]);
            } else {
                const v4f a4 = stash[row * 16 + (q ^ (row & 15))];
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = act_fast<ACT>(sg * a4[i] + b4[i]) * inv;
            }
        };
        auto for_each_fm = [&](auto&& f) {
            f(act_tag<0>{}); f(act_tag<1>{}); f(act_tag<2>{}); f(act_tag<3>{});
            f(act_tag<4>{}); f(act_tag<5>{}); f(act_tag<6>{}); f(act_tag<7>{});
        };
        if (vec_ok && rows == 256 && cols == (GATED ? 128 : 256)) {
            auto whole = [&](auto out_tag, auto act) {
                constexpr int OUT = decltype(out_tag)::value, ACT = decltype(act)::value;
                constexpr int OSZ = OUT == EPARA_BF16 ? 2 : 1;
                typedef float v2f __attribute__((ext_vector_type(2)));
                typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
                EPARA_GLOBAL char* ybase = as_global<char>(ga.Y) + (static_cast<size_t>(m0) * N + n0 + wave * WCOLS) * OSZ;   // uniform
                const uint32_t lane_off = static_cast<uint32_t>((rr * N + 4 * q) * OSZ);
                for_each_fm([&](auto fm_tag) {
                    constexpr int fm = decltype(fm_tag)::value;
                    park(fm_tag);
#pragma unroll
                    for (int it = 0; it < 32 / RPI; ++it) {
                        float v[4];
                        finish(act, it * RPI + rr, v);
                        EPARA_GLOBAL char* y = ybase + static_cast<size_t>(fm * 32 + it * RPI) * N * OSZ + lane_off;
                        if constexpr (OUT == EPARA_BF16) {
                            v2u pk;
                            pk[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector((v2f{v[0], v[1]}), v2bf));
                            pk[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector((v2f{v[2], v[3]}), v2bf));
                            put<WT>(reinterpret_cast<EPARA_GLOBAL v2u*>(y), pk);
                        } else {
                            put<WT>(reinterpret_cast<EPARA_GLOBAL uint32_t*>(y), f32x4_to_e4m3(v[0], v[1], v[2], v[3]));
                        }
                    }
                });
            };
            auto by_out = [&](auto act) {
                if (DT == EPARA_BF16 || out_dtype == EPARA_BF16) whole(act_tag<EPARA_BF16>{}, act);
                else if constexpr (DT != EPARA_BF16)              whole(act_tag<EPARA_FP8_E4M3>{}, act);
            };
            if constexpr (GATED) by_out(act_tag<EPARA_ACT_SILU>{});
            else                 with_act(ga.act, by_out);
        } else {
            const int act = ga.act;
            for_each_fm([&](auto fm_tag) {
                constexpr int fm = decltype(fm_tag)::value;
                if (fm * 32 < rows) {
                    park(fm_tag);
#pragma unroll 1
                    for (int it = 0; it < 32 / RPI; ++it) {
                        const int row = it * RPI + rr;
                        if (fm * 32 + row < rows && nl < cols) {
                            float v[4];
                            if constexpr (GATED) finish(act_tag<EPARA_ACT_SILU>{}, row, v);
                            else if (act == EPARA_ACT_RELU)      finish(act_tag<EPARA_ACT_RELU>{}, row, v);
                            else if (act == EPARA_ACT_GELU_ERF)  finish(act_tag<EPARA_ACT_GELU_ERF>{}, row, v);
                            else if (act == EPARA_ACT_GELU_TANH) finish(act_tag<EPARA_ACT_GELU_TANH>{}, row, v);
                            else if (act == EPARA_ACT_SILU)      finish(act_tag<EPARA_ACT_SILU>{}, row, v);
                            else                                 finish(act_tag<EPARA_ACT_NONE>{}, row, v);
                            store4<WT>(ga.Y, out_dtype, static_cast<size_t>(m0 + fm * 32 + row), n0 + nl, N, v, cols - nl, vec_ok);
                        }
                    }
                }
            });
        }
        if constexpr (CHAIN) chain_done(*chain, cw.tl.group);
        w_next(cw);
        if (cw.t < 0) break;
    }
    wait_vmcnt<0>();                                             // the loads past the end of the run
    __syncthreads();
    // first slot after the run: the next non-idle slot of this workgroup or the end
    long s = cw.slot;
    if (s < n_slots && order[s] < 0)
        for (s += stride; s < n_slots && order[s] < 0; s += stride) {}
    return s;
}

// The visit that counted last at a split panel tile: adds the NP parts (row-major 256 x 256 fp32 each) in index
// order, whoever wrote them last, and runs the plain epilogue.  Lane l of wave w takes columns 4 l .. 4 l + 3 of the
// rows w, w + 4, w + 8, ...; eight rows at a time: all their parts are asked for first (16-byte device-scope loads
// into registers), then added and stored, so a batch costs one trip to memory.
template <int DT, int NP>
__device__ __forceinline__ void panel_split_finish_n(const epara_group_args& ga, const epara_tile& tl, int out_dtype, int pslot,
                                                     int tid, const split_ctx* sp)
{
    constexpr int R = 8;                                         // rows per lane and batch
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c4 = 4 * lane;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        panel_partials(*sp) + static_cast<size_t>(pslot) * SPLIT_MAX_PARTS * PANEL_SPLIT_STRIDE, 0, -1, 0x00020000);
    const bool vec_ok = (ga.N & 3) == 0;
    float b4[4] = {0.f, 0.f, 0.f, 0.f};
    if (ga.bias) {
#pragma unroll
        for (int i = 0; i < 4; ++i) if (c4 + i < tl.cols) b4[i] = as_global<float>(ga.bias)[tl.n0 + c4 + i];
    }
    const float sg = ga.scale, inv = ga.out_inv_scale;
    auto run = [&](auto act) {
        constexpr int ACT = decltype(act)::value;
        for (int rb = wave; rb < tl.rows; rb += 4 * R) {
            v4i in[R][NP];
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const int row = min(rb + 4 * k, tl.rows - 1);
#pragma unroll
                for (int pt = 0; pt < NP; ++pt)
                    in[k][pt] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane * 16, pt * PANEL_SPLIT_STRIDE + row * 1024, 16);   // 16: device scope (sc1)
            }
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const int row = rb + 4 * k;
                v4f sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int pt = 0; pt < NP; ++pt) sum += __builtin_bit_cast(v4f, in[k][pt]);
                if (row < tl.rows && c4 < tl.cols) {
                    float v[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = act_fast<ACT>(sg * sum[i] + b4[i]) * inv;
                    store4<false>(ga.Y, out_dtype, static_cast<size_t>(tl.m0 + row), tl.n0 + c4, ga.N, v, tl.cols - c4, vec_ok);
                }
            }
        }
    };
    with_act(ga.act, run);
}

template <int DT>
__device__ __forceinline__ void panel_split_finish(const epara_group_args& ga, const epara_tile& tl, int out_dtype, int pslot, int nparts,
                                                   int tid, const split_ctx* sp, char*)
{
    if (nparts == 2)      panel_split_finish_n<DT, 2>(ga, tl, out_dtype, pslot, tid, sp);
    else if (nparts == 3) panel_split_finish_n<DT, 3>(ga, tl, out_dtype, pslot, tid, sp);
    else                  panel_split_finish_n<DT, 4>(ga, tl, out_dtype, pslot, tid, sp);
}

}  // namespace

#endif
