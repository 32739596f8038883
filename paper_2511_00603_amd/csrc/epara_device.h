// Device helpers shared by the kernels of libepara (gfx950): activations, matrix-core wrappers,
// output stores and casts, the epilogue of one accumulator quad, wait-count helpers and the
// completion counters that order the phases of a chain.
//
// MFMA orientation.  D = A*B with A = weight fragments and B = activation fragments, both as
// 16-byte "k-chunks": a lane feeds chunk q of weight column / activation row r to A and B and
// receives four consecutive output columns of one row per accumulator quad -- what a row-major
// store wants.  Only the pairing of A and B chunks matters for the sum, so the same code
// serves bf16 (8 values per chunk) and fp8 (16 values per chunk).
//   16x16x32: lane = (r = lane%16, q = lane/16), D[n = 4q+i][m = r]
//   32x32x16: lane = (r = lane%32, h = lane/32), D[n = 8(v/4) + 4h + v%4][m = r], v = 0..15
#ifndef EPARA_DEVICE_H
#define EPARA_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "epara.h"
#include "epara_cast.h"

namespace {

using epara_cast::f32_to_bf16;
using epara_cast::f32_to_e4m3;
using epara_cast::f32x4_to_e4m3;

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int NT = 256;                 // threads per workgroup (4 waves, one per SIMD)
constexpr int BIAS_LDS_OFFSET = 131072;  // after the operand buffers: 256 floats, the bias of a panel tile
constexpr int LDS_BYTES = 163840;          // the whole LDS of a compute unit (one workgroup per unit)
constexpr int RING_LDS_OFFSET = 65536;   // streaming tiles: partial sums below, the waves' activation rings above
constexpr int F32_BM = 64, F32_BN = 64, F32_BK = 64, F32_NT = 256;
constexpr int F32_PER = F32_BM * F32_BK / F32_NT;      // elements of X (and of W) a thread stages per K step

// ------------------------------------------------------------------ small device helpers

template <int ACT>
__device__ __forceinline__ float act_apply(float z)
{
    if constexpr (ACT == EPARA_ACT_RELU)           return z > 0.f ? z : 0.f;
    else if constexpr (ACT == EPARA_ACT_GELU_ERF)  return 0.5f * z * (1.f + erff(z * 0.70710678118654752f));
    else if constexpr (ACT == EPARA_ACT_GELU_TANH) return 0.5f * z * (1.f + tanhf(0.79788456080286536f * (z + 0.044715f * z * z * z)));
    else if constexpr (ACT == EPARA_ACT_SILU)      return z / (1.f + expf(-z));
    else                                           return z;
}

// Calls f(tag) with tag an integral_constant of the runtime activation, so that the unrolled
// epilogues are compiled once per activation instead of carrying a switch per element.
template <int V> struct act_tag { static constexpr int value = V; };
template <class F>
__device__ __forceinline__ void with_act(int act, F&& f)
{
    switch (act) {
    case EPARA_ACT_RELU:      f(act_tag<EPARA_ACT_RELU>{}); break;
    case EPARA_ACT_GELU_ERF:  f(act_tag<EPARA_ACT_GELU_ERF>{}); break;
    case EPARA_ACT_GELU_TANH: f(act_tag<EPARA_ACT_GELU_TANH>{}); break;
    case EPARA_ACT_SILU:      f(act_tag<EPARA_ACT_SILU>{}); break;
    default:                  f(act_tag<EPARA_ACT_NONE>{}); break;
    }
}

// The same activations for the 16- and 8-bit paths, whose outputs keep 8 or 3 mantissa bits: the
// exponential and the reciprocal are the hardware's (about 1 ulp in fp32) instead of the exactly
// rounded library forms, and the normal distribution function of the erf form of GELU is a logistic
// function of an odd polynomial, Phi(z) ~ 1 / (1 + exp(-z (a + b z^2 + c z^4))), fitted to the erf form
// (not to the tanh form) on |z| <= 8, where z^2 is clamped: |z Phi(z) - GELU(z)| < 2.6e-5 for all z.
// One wave per SIMD has nobody to overlap an epilogue with, so its instruction count is paid in full
// on every tile: this form is 7 plain and 2 transcendental instructions, the Abramowitz-Stegun
// rational-times-Gaussian erf it replaces took 17 and 2.
__device__ __forceinline__ float fast_logistic(float t)      // 1 / (1 + e^-t)
{
    return __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * t));
}
template <int ACT>
__device__ __forceinline__ float act_fast(float z)
{
    if constexpr (ACT == EPARA_ACT_RELU)           return fmaxf(z, 0.f);
    else if constexpr (ACT == EPARA_ACT_GELU_ERF) {
        // the coefficients carry the factor -log2(e): the exponential is the hardware's base-2 one
        const float z2 = fminf(z * z, 64.f);
        const float u = z * (-2.3011138f + z2 * (-0.10678257f + z2 * 0.0010153757f));
        return z * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(u));
    }
    else if constexpr (ACT == EPARA_ACT_GELU_TANH) // 0.5 z (1 + tanh u) = z / (1 + e^-2u)
        return z * fast_logistic(1.5957691216057308f * (z + 0.044715f * z * z * z));
    else if constexpr (ACT == EPARA_ACT_SILU)      return z * fast_logistic(z);
    else                                           return z;
}

template <int DT>
__device__ __forceinline__ void mma(v4f& c, const v4i& a, const v4i& b)
{
    if constexpr (DT == EPARA_BF16) {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    } else {
        typedef long v2l __attribute__((ext_vector_type(2)));
        const v2l al = __builtin_bit_cast(v2l, a), bl = __builtin_bit_cast(v2l, b);
        c = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(al[0], bl[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(al[1], bl[1], c, 0, 0, 0);
    }
}

// 32x32 accumulate of one 16-byte chunk pair per lane (bf16: K = 16; fp8: two K = 16 halves).
template <int DT>
__device__ __forceinline__ void mma32(v16f& c, const v4i& a, const v4i& b)
{
    if constexpr (DT == EPARA_BF16) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    } else {
        typedef long v2l __attribute__((ext_vector_type(2)));
        const v2l al = __builtin_bit_cast(v2l, a), bl = __builtin_bit_cast(v2l, b);
        c = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(al[0], bl[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(al[1], bl[1], c, 0, 0, 0);
    }
}

// Pointers read from the argument table are generic; the kernels know they are global memory.
#define EPARA_GLOBAL __attribute__((address_space(1)))
typedef const EPARA_GLOBAL char* gcptr;
template <class T>
__device__ __forceinline__ const EPARA_GLOBAL T* as_global(const void* p) { return (const EPARA_GLOBAL T*)p; }
template <class T>
__device__ __forceinline__ EPARA_GLOBAL T* as_global(void* p) { return (EPARA_GLOBAL T*)p; }

__device__ __forceinline__ v4i ld16(gcptr p) { return *reinterpret_cast<const EPARA_GLOBAL v4i*>(p); }

// Output stores.  WT ("write through"): the outputs of a chain are read by other workgroups of the
// same kernel, possibly on another compute die with its own L2; stored as device-scope atomic
// (relaxed) stores they go through to memory at once, and the producer's release needs no
// write-back of its whole L2 -- which costs microseconds per workgroup and tile group.
template <bool WT, class T>
__device__ __forceinline__ void put(EPARA_GLOBAL T* p, T v)
{
    if constexpr (WT) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *p = v;
}
template <bool WT>
__device__ __forceinline__ void put(EPARA_GLOBAL v2u* p, v2u v)
{
    if constexpr (WT) __hip_atomic_store(reinterpret_cast<EPARA_GLOBAL uint64_t*>(p), __builtin_bit_cast(uint64_t, v),
                                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *p = v;
}

// Stores up to four consecutive outputs of one row, starting at column n (a multiple of 4).
template <bool WT>
__device__ __forceinline__ void store4(void* Y, int out_dtype, size_t m, int n, int N, const float* v, int valid, bool vec_ok)
{
    const size_t e = m * static_cast<size_t>(N) + n;
    if (out_dtype == EPARA_BF16) {
        EPARA_GLOBAL uint16_t* y = as_global<uint16_t>(Y) + e;
        if (vec_ok && valid >= 4) {
            typedef float v2f __attribute__((ext_vector_type(2)));
            typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
            v2u pk;                               // round to nearest even in hardware, two values per instruction
            pk[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector((v2f{v[0], v[1]}), v2bf));
            pk[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector((v2f{v[2], v[3]}), v2bf));
            put<WT>(reinterpret_cast<EPARA_GLOBAL v2u*>(y), pk);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (i < valid) put<WT>(y + i, static_cast<uint16_t>(f32_to_bf16(v[i])));
        }
    } else {  // EPARA_FP8_E4M3
        EPARA_GLOBAL uint8_t* y = as_global<uint8_t>(Y) + e;
        if (vec_ok && valid >= 4) {
            put<WT>(reinterpret_cast<EPARA_GLOBAL uint32_t*>(y), f32x4_to_e4m3(v[0], v[1], v[2], v[3]));
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (i < valid) put<WT>(y + i, static_cast<uint8_t>(f32_to_e4m3(v[i])));
        }
    }
}

// Epilogue of one accumulator quad (plain groups): the lane holds columns nl..nl+3 of row ml.
// `bias` points at the bias of column n0 (global memory for streaming tiles; panel tiles stage the
// tile's 256 bias values in LDS first, because a global load inside the store loop would make
// every iteration wait for all earlier stores: loads and stores share one in-order counter).
template <int ACT, bool WT, class BiasPtr>
__device__ __forceinline__ void finish_plain(const epara_group_args& ga, int out_dtype, const v4f& a, BiasPtr bias,
                                             int m0, int ml, int rows, int n0, int nl, int cols, bool vec_ok)
{
    if (ml >= rows || nl >= cols) return;
    const int valid = cols - nl;
    float v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float b = 0.f;
        if (bias && i < valid) b = bias[nl + i];
        v[i] = act_fast<ACT>(ga.scale * a[i] + b) * ga.out_inv_scale;
    }
    store4<WT>(ga.Y, out_dtype, static_cast<size_t>(m0 + ml), n0 + nl, ga.N, v, valid, vec_ok);
}

// Epilogue of a gate/up fragment pair (EPARA_ACT_SWIGLU groups).
template <bool WT>
__device__ __forceinline__ void finish_gated(const epara_group_args& ga, int out_dtype, const v4f& g, const v4f& u,
                                             int m0, int ml, int rows, int n0, int nl, int cols, bool vec_ok)
{
    if (ml >= rows || nl >= cols) return;
    float v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = act_fast<EPARA_ACT_SILU>(ga.scale * g[i]) * (ga.scale2 * u[i]) * ga.out_inv_scale;
    store4<WT>(ga.Y, out_dtype, static_cast<size_t>(m0 + ml), n0 + nl, ga.N, v, cols - nl, vec_ok);
}

typedef __attribute__((address_space(3))) char* ldsptr;
typedef const __attribute__((address_space(3))) v4i* lds_v4i;

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N < 64, "vmcnt is 6 bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);    // expcnt / lgkmcnt untouched
}
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// ------------------------------------------------------------------ chains of launches in one kernel
//
// Completion counters in device memory order the phases of a chain: a workgroup adds the number of
// tiles of a group it has stored to that group's counter (after a device-scope release: the
// compute dies have separate L2 caches), and a tile whose group reads that output first polls the
// counter until it holds the group's tile count, then acquires.  All fields are the same in every
// thread of the workgroup, so every thread takes the same barriers.
constexpr int CHAIN_HEADER_WORDS = 4;    // [0] error flag, [1] workgroups that have left the kernel

struct chain_ctx {
    const epara_chain_wait* waits;   // of the current phase, or null
    uint32_t* ws;                    // workspace: header, then the counters
    uint32_t spin_limit;
    int counter_base;                // of the current phase
    int pend_group[2], pend_n[2];    // stored tiles not yet counted, for up to two groups
    int ok_group;                    // the group whose wait was passed last
};

__device__ __forceinline__ void chain_flush(chain_ctx& c)
{
    if (c.pend_n[0] == 0 && c.pend_n[1] == 0) return;
    // The tiles were stored with write-through stores (put<true>): once every wave has seen its stores
    // complete they are in memory, and the counts may follow.  A device-scope release fence would do
    // the same and also write back the die's whole L2, which is what this path avoids.
    wait_vmcnt<0>();                                             // this wave's stores are done
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            if (c.pend_n[i] > 0) {
                // the returned value is asked for so that the wave can wait for the add itself (chain_exit)
                const uint32_t before = __hip_atomic_fetch_add(c.ws + CHAIN_HEADER_WORDS + c.counter_base + c.pend_group[i],
                                                               static_cast<uint32_t>(c.pend_n[i]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                asm volatile("" :: "v"(before));
            }
    }
    c.pend_n[0] = c.pend_n[1] = 0;
}

// A finished tile is counted at once if its group is one of the two being collected; a third group
// publishes the other two first.  (Publishing drains the wave's loads in flight, so it is done
// rarely: a workgroup's list holds the tiles of a group together.)
__device__ __forceinline__ void chain_done(chain_ctx& c, int group)
{
    if (c.pend_n[0] > 0 && c.pend_group[0] == group) { ++c.pend_n[0]; return; }
    if (c.pend_n[1] > 0 && c.pend_group[1] == group) { ++c.pend_n[1]; return; }
    if (c.pend_n[0] > 0 && c.pend_n[1] > 0) chain_flush(c);
    const int i = c.pend_n[0] == 0 ? 0 : 1;
    c.pend_group[i] = group;
    c.pend_n[i] = 1;
}

// True if a tile of `group` has to wait (or may have to) before its input can be read.
__device__ __forceinline__ bool chain_must_wait(const chain_ctx& c, int group)
{
    return c.waits != nullptr && group != c.ok_group && c.waits[group].counter >= 0 && c.waits[group].need > 0;
}

// No cache is invalidated after the wait.  A line of the produced tensor can only be in this die's
// L2 or this unit's L1 if it was read, and inside this kernel it is read only by tiles that have
// passed this wait, i.e. after all of it was written through to memory; lines cached by an earlier
// kernel are dropped at the kernel boundary.  (A device-scope acquire would invalidate the die's
// whole L2 at every wait, and with it the activation rows that the tiles of a group share.)
__device__ __forceinline__ void chain_wait(chain_ctx& c, int group)
{
    if (!chain_must_wait(c, group)) { c.ok_group = group; return; }
    const epara_chain_wait w = c.waits[group];
    if (threadIdx.x == 0) {
        const uint32_t* ctr = c.ws + CHAIN_HEADER_WORDS + w.counter;
        uint32_t polls = 0;
        while (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < static_cast<uint32_t>(w.need)) {
            if (++polls >= c.spin_limit) {                       // bounded: report and go on, the kernel always ends
                __hip_atomic_store(c.ws, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            // once any wait has run out the chain's results are lost anyway: nobody waits any longer
            if ((polls & 63u) == 0 && __hip_atomic_load(c.ws, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) break;
            __builtin_amdgcn_s_sleep(8);
        }
    }
    __syncthreads();                                             // nobody reads the produced rows before the count was seen
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    c.ok_group = group;
}

// The last workgroup to leave puts the counters back to zero for the next chain on this workspace
// (the kernel boundary orders these stores before that chain).
__device__ __forceinline__ void chain_exit(chain_ctx& c, int n_counters)
{
    chain_flush(c);
    wait_vmcnt<0>();                                             // my counter adds have been performed (they return a value)
    __syncthreads();
    if (threadIdx.x == 0) {
        // nothing of this workgroup is still on its way to a counter when it is counted as gone, so the
        // zeroing below cannot be overtaken by a late add
        const uint32_t left = __hip_atomic_fetch_add(c.ws + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (left + 1 == gridDim.x) {
            for (int i = 0; i < n_counters; ++i)
                __hip_atomic_store(c.ws + CHAIN_HEADER_WORDS + i, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(c.ws + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

constexpr int N_STREAM_CLASSES = 3;

// An entry of the visit order: bits 0..23 the tile, bits 24..27 which part of K this visit multiplies,
// bits 28..30 the number of parts minus one (0: the whole K, the common case); negative: idle.
__device__ __forceinline__ int order_tile(int o)  { return o & 0xFFFFFF; }
__device__ __forceinline__ int order_part(int o)  { return (o >> 24) & 15; }
__device__ __forceinline__ int order_parts(int o) { return ((o >> 28) & 7) + 1; }

// Streaming tiles whose K is split over several visits (possibly of different workgroups) meet in a
// device workspace: one arrival counter per split tile, then, 256-byte aligned, SPLIT_MAX_PARTS x
// SPLIT_STRIDE bytes of partial sums per split tile.  The visit that arrives last adds the parts in index order and
// runs the epilogue, so the result does not depend on who that is.
constexpr int SPLIT_STRIDE = EPARA_SPLIT_STRIDE, SPLIT_MAX_PARTS = EPARA_SPLIT_MAX_PARTS;
constexpr int PANEL_SPLIT_STRIDE = EPARA_PANEL_SPLIT_STRIDE;
// n_split streaming tiles, then n_panel panel tiles (the tiles first_panel ... of the tile table): counters in that
// order, then the streaming tiles' partial sums, then the panel tiles'.
struct split_ctx { uint32_t* ws; int n_split; int n_panel; int first_panel; };
__device__ __forceinline__ char* split_partials(const split_ctx& sp)
{
    return reinterpret_cast<char*>(sp.ws) + (((sp.n_split + sp.n_panel) * 4 + 255) & ~255);
}
__device__ __forceinline__ char* panel_partials(const split_ctx& sp)
{
    return split_partials(sp) + static_cast<size_t>(sp.n_split) * SPLIT_MAX_PARTS * SPLIT_STRIDE;
}
__device__ __forceinline__ void split_put(char* at, const v4f& v)     // through to memory: another die reads it
{
    typedef unsigned long long u64;
    const u64 lo = (static_cast<u64>(__float_as_uint(v[1])) << 32) | __float_as_uint(v[0]);
    const u64 hi = (static_cast<u64>(__float_as_uint(v[3])) << 32) | __float_as_uint(v[2]);
    __hip_atomic_store(reinterpret_cast<u64*>(at), lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(reinterpret_cast<u64*>(at) + 1, hi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The same store as one 16-byte instruction (the compiler has no 16-byte atomic store to offer): whole 256-byte row
// pieces leave a quarter wave at once.  Nothing is returned, so only the explicit wait before a visit is counted
// has to know about it; loads and stores complete in issue order, which keeps every other wait conservative.
// A store of more than 8 bytes reads its data registers a cycle after it issues, and the compiler's hazard
// check does not look inside an asm statement: the wait state that keeps the next instruction from
// overwriting them is part of the statement.
__device__ __forceinline__ void split_put16(char* at, const v4f& v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(at), "v"(v) : "memory");
}
__device__ __forceinline__ v4f split_get(const char* at)
{
    typedef unsigned long long u64;
    const u64 lo = __hip_atomic_load(reinterpret_cast<const u64*>(at), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const u64 hi = __hip_atomic_load(reinterpret_cast<const u64*>(at) + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return v4f{__uint_as_float(static_cast<uint32_t>(lo)), __uint_as_float(static_cast<uint32_t>(lo >> 32)),
               __uint_as_float(static_cast<uint32_t>(hi)), __uint_as_float(static_cast<uint32_t>(hi >> 32))};
}

// The visits a workgroup has made to tiles whose K is split, not yet counted at the tiles' counters: lane i
// of `slots` / `entries` holds the i-th (the same in every wave).  Counting is put off to the end of the
// workgroup's list, where one atomic instruction does it for all of them and nothing waits for it in the
// middle of a weight stream.
struct split_pending {
    int count;
    int slots;             // the tile's workspace slot | (parts - 1) << 28
    int entries;           // the visit's entry of the order
};

}  // namespace

#endif
