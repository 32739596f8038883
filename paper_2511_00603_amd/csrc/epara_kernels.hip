// Device half of libepara: persistent grouped forward kernels for gfx950 (MI355X).
//
// One launch serves every co-located service (the MT operator of Sec. 3.1): persistent
// workgroups walk a device tile table in a precomputed visit order; a tile is either
//   - "big":    256 rows x 256 columns of one group, both operands LDS-staged by direct loads,
//               32x32x16 MFMA (fp8: 32x32x64), or
//   - "skinny": a whole batch of <= 64 rows x 32 .. 128 columns, weights streamed from HBM
//               straight into 16x16x32 MFMA operand registers, activations through a small
//               LDS ring per wave, K split over the four waves of the workgroup.
// Bias, activation, SwiGLU gating, fp8 scales and the output cast are fused in the epilogue.
// A workgroup is four waves, one per SIMD, so a wave may use the whole 512-entry register
// file: 256 accumulators for a 128 x 128 wave tile plus double-buffered operand fragments.
//
// MFMA orientation.  D = A*B with A = weight fragments and B = activation fragments, both as
// 16-byte "k-chunks": a lane feeds chunk q of weight column / activation row r to A and B and
// receives four consecutive output columns of one row per accumulator quad -- what a row-major
// store wants.  Only the pairing of A and B chunks matters for the sum, so the same code
// serves bf16 (8 values per chunk) and fp8 (16 values per chunk).
//   16x16x32: lane = (r = lane%16, q = lane/16), D[n = 4q+i][m = r]
//   32x32x16: lane = (r = lane%32, h = lane/32), D[n = 8(v/4) + 4h + v%4][m = r], v = 0..15
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <cstring>
#include <vector>

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
// rounded library forms, and erf is the rational-times-Gaussian approximation of Abramowitz and
// Stegun (7.1.26, absolute error below 1.5e-7).  One wave per SIMD has nobody to overlap an
// epilogue with, so its instruction count is paid in full on every tile.
__device__ __forceinline__ float fast_logistic(float t)      // 1 / (1 + e^-t)
{
    return __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * t));
}
template <int ACT>
__device__ __forceinline__ float act_fast(float z)
{
    if constexpr (ACT == EPARA_ACT_RELU)           return fmaxf(z, 0.f);
    else if constexpr (ACT == EPARA_ACT_GELU_ERF) {
        const float x = fabsf(z) * 0.70710678118654752f;
        const float t = __builtin_amdgcn_rcpf(1.f + 0.3275911f * x);
        const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
        const float tail = poly * __builtin_amdgcn_exp2f(-1.4426950408889634f * x * x);   // 1 - erf(x)
        return 0.5f * z * (z < 0.f ? tail : 2.f - tail);
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

// ------------------------------------------------------------------ big tiles (LDS + MFMA)

// One 256 x 256 output tile (gated: 256 rows x 128 hidden columns, i.e. 128 gate + 128 up
// weight columns).  K advances in stages of 64 bytes per row (one packed weight fragment per
// column block).  All operands reach the LDS by direct global->LDS loads (no staging registers):
//   W: four stage buffers of 16 KiB (16 column blocks x 1 KiB, a verbatim image of the packed
//      fragments), refilled four stages ahead;
//   X: two buffers of 32 KiB, each holding TWO stages (256 rows x 128 B), refilled two stages
//      ahead.  A load instruction then covers whole 128-byte lines (8 rows x 128 B per wave
//      instruction); fetching 64-byte half lines costs a full line slot in the L1 each.
//      16-byte chunk c of row `row` is stored at chunk c ^ ((row/2)%8), so the 16 rows that one
//      quarter of a ds_read_b128 touches fall into 16 different bank groups; a direct load writes
//      1 KiB of consecutive LDS, so lane l fetches the global chunk that belongs at position l.
// Rows past the batch and column blocks past N are clamped to the last valid one (they only
// feed outputs that are never stored).  In a ragged last stage the X chunks past K are clamped
// to chunk 0 of the buffer: the packed weights are zero there, so the products vanish.  Loads past
// the end of K re-load the last data into buffers nobody reads, which keeps the loop free of
// branches.
//
// A stage is two 32x32x16 steps.  Operand fragments are double-buffered in registers: the
// reads of step s+1 are issued between the MFMAs of step s.  In the middle of stage kt every
// wave waits for its own loads of stage kt+1, a workgroup barrier makes all parts visible (and
// proves that every wave has finished reading stage kt), and the freed buffers are refilled:
// W stage kt+4 always, X stages kt+3 and kt+4 when kt is odd.  Loads complete in issue order, so
// "my loads of stage kt+1 have landed" is a bound on the number of loads still in flight: 16
// in an even stage (two W stages and an X pair were issued later), 4 in an odd one.
typedef __attribute__((address_space(3))) char* ldsptr;
typedef const __attribute__((address_space(3))) v4i* lds_v4i;

constexpr int XBUF_BYTES = 32768;        // one X buffer: 256 rows x 128 B = two stages
constexpr int WBUF_BYTES = 16384;        // one W stage: 16 column blocks x 1 KiB
constexpr int W_LDS_OFFSET = 2 * XBUF_BYTES;

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N < 64, "vmcnt is 6 bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);    // expcnt / lgkmcnt untouched
}
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// `advance` is called three times, well apart (after the first loads are issued, when the multiply
// loop starts, when it ends): the caller uses it to fetch the records of its next tile, one
// dependent scalar load per call, so that their latencies pass under this tile.
template <int DT, bool GATED, bool WT, class Advance>
__device__ __forceinline__ void big_tile(const epara_group_args& ga, int out_dtype,
                                         int m0, int n0, int rows, int cols, char* lds, Advance&& advance)
{
    constexpr int ESZ = DT == EPARA_BF16 ? 2 : 1;
    constexpr int EPC = 16 / ESZ;   // elements per 16-byte chunk
    constexpr int KF = 4 * EPC;     // K elements per stage (one weight fragment)
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r32 = lane & 31, h = lane >> 5;
    const int wn = wave & 1, wm = wave >> 1;
    const int K = ga.K, N = ga.N;
    const int KS = (K + KF - 1) / KF;
    const int KD = (KS + 1) >> 1;                               // X stage pairs
    const int NB = (N + 15) >> 4;
    ldsptr l3 = (ldsptr)lds;

    // --- direct-load descriptors: this wave fills X rows [64 wave, 64 wave + 64) and W blocks 4 wave .. 4 wave + 3
    const int tail_k = K - (KD - 1) * 2 * KF;                   // elements in the last stage pair, 1..2KF
    uint32_t xoff[8], xoff_tail[8], woff[4];
#pragma unroll
    for (int j = 0; j < 8; ++j) {                               // instruction j: rows 64 wave + 8 j .. + 7, lane -> (row l/8, slot l%8)
        const int row_in_tile = 64 * wave + 8 * j + (lane >> 3);
        const int chunk = (lane & 7) ^ ((4 * (j & 1) + (lane >> 4)) & 7);      // = slot ^ ((row/2)%8)
        const int chunk_tail = (chunk * EPC < tail_k) ? chunk : 0;
        const int row = min(row_in_tile, rows - 1);
        xoff[j] = static_cast<uint32_t>((row * K + chunk * EPC) * ESZ);
        xoff_tail[j] = static_cast<uint32_t>((row * K + chunk_tail * EPC) * ESZ);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int nbrel = (GATED ? ((4 * wave) & 7) : 4 * wave) + j;
        const int nb = min(nbrel, NB - 1 - (n0 >> 4));
        woff[j] = static_cast<uint32_t>((nb * KS * 64 + lane) * 16);
    }

    // Direct loads go through buffer descriptors spanning the whole address space (every offset
    // below is already clamped to valid memory): a wave issues this form a little faster than the
    // flat-encoded one, and it leaves the compiler's count of outstanding loads exact.
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(static_cast<const char*>((GATED && wave >= 2) ? ga.W2 : ga.W)) + static_cast<size_t>(n0 >> 4) * KS * 1024, 0, -1, 0x00020000);
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(static_cast<const char*>(ga.X)) + static_cast<size_t>(m0) * K * ESZ, 0, -1, 0x00020000);
    // direct loads, one instruction at a time so that they can be spread between the MFMAs
    auto issue_w1 = [&](int kt_unclamped, int j) {
        const int buf = W_LDS_OFFSET + (kt_unclamped & 3) * WBUF_BYTES + 4 * wave * 1024;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(wrsrc, (__attribute__((address_space(3))) void*)(l3 + buf + j * 1024), 16,
                                                 woff[j], min(kt_unclamped, KS - 1) * 1024, 0, 0);
    };
    auto issue_x1 = [&](int kd_unclamped, int j) {
        const int buf = (kd_unclamped & 1) * XBUF_BYTES + 8 * wave * 1024;
        const int kd = min(kd_unclamped, KD - 1);
        const bool tail = kd == KD - 1;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(xrsrc, (__attribute__((address_space(3))) void*)(l3 + buf + j * 1024), 16,
                                                 tail ? xoff_tail[j] : xoff[j], kd * 128, 0, 0);
    };
    auto issue_w = [&](int kt) {
#pragma unroll
        for (int j = 0; j < 4; ++j) issue_w1(kt, j);
    };
    auto issue_x = [&](int kd) {
#pragma unroll
        for (int j = 0; j < 8; ++j) issue_x1(kd, j);
    };

    // --- fragment read offsets
    //   X fragment fm of step s16 = 0..3 of a stage pair: rows wm*128 + fm*32 + r32, chunk 2 s16 + h
    //   W fragment fn = column blocks (2 fn, 2 fn + 1) of the wave's eight: lane r32 -> block r32/16, column r32%16
    const int sw = (r32 >> 1) & 7;
    int xf_off[4];
#pragma unroll
    for (int s16 = 0; s16 < 4; ++s16) xf_off[s16] = (wm * 128 + r32) * 128 + (((2 * s16 + h) ^ sw) << 4);   // + fm * 4096
    const int wf_off = W_LDS_OFFSET + ((GATED ? wn * 4 : wn * 8) + (r32 >> 4)) * 1024 + (h * 16 + (r32 & 15)) * 16;   // + blk*1024 + s*512

    v16f acc[4][4];
#pragma unroll
    for (int fn = 0; fn < 4; ++fn)
#pragma unroll
        for (int fm = 0; fm < 4; ++fm)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[fn][fm][v] = 0.f;

    typedef __attribute__((address_space(3))) float* lds_float;
    lds_float bias_tile = (lds_float)(l3 + BIAS_LDS_OFFSET);
    float my_bias = 0.f;                   // fetched before the direct loads start, so that waiting for it is free
    if (!GATED && ga.bias && n0 + tid < N) my_bias = as_global<float>(ga.bias)[n0 + tid];
    wait_vmcnt<0>();                       // nothing of the previous tile is still landing in the LDS
    __syncthreads();                       // and nobody still reads it
    if (!GATED) bias_tile[tid] = my_bias;   // zeros when the group has no bias: the epilogue adds it unconditionally
    issue_w(0); issue_w(1); issue_x(0); issue_w(2); issue_w(3); issue_x(1);
    advance();
    wait_vmcnt<16>();                      // W0, W1, X(0,1) have landed
    __builtin_amdgcn_s_barrier();
    advance();
    if constexpr (DT == EPARA_BF16) {
        v4i wf[2][4], xf[2][4];
        // Fragment i = 0..7 of step (kt, s2), in the order the next half's MFMAs need them:
        // W0, X0, X1, X2, X3, W1, W2, W3.  kt_par = kt & 1 must be a compile-time value.
        auto read_frag = [&](int kt, int kt_par, int s2, int set, int i) {
            if (i == 0 || i >= 5) {
                const int fn = i == 0 ? 0 : i - 4;
                const int blk = GATED ? (fn < 2 ? 2 * fn : 8 + 2 * (fn - 2)) : 2 * fn;   // gate blocks 0..3, up blocks 8..11 (+ 4 wn)
                wf[set][fn] = *reinterpret_cast<lds_v4i>(l3 + (kt & 3) * WBUF_BYTES + wf_off + blk * 1024 + s2 * 512);
            } else {
                const int fm = i - 1;
                xf[set][fm] = *reinterpret_cast<lds_v4i>(l3 + ((kt >> 1) & 1) * XBUF_BYTES + xf_off[2 * kt_par + s2] + fm * 4096);
            }
        };
        // Half a stage: 16 MFMAs on register set `set` in eight groups of two; after each of the first
        // four groups two fragments of the next step are read into the other set, and after each
        // group up to two direct loads are issued.  The
        // scheduling barriers pin this interleaving: one wave per SIMD has nobody else to hide a stall.
        auto half = [&](int set, int kt_read, int par_read, int s2_read, int kt_w, int kd_x) {
    #pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int fn = i >> 1, fm = 2 * (i & 1);
                mma32<DT>(acc[fn][fm], wf[set][fn], xf[set][fm]);
                mma32<DT>(acc[fn][fm + 1], wf[set][fn], xf[set][fm + 1]);
                if (i < 4) {                    // all eight reads early: the last MFMAs of the half cover their latency
                    read_frag(kt_read, par_read, s2_read, set ^ 1, 2 * i);
                    read_frag(kt_read, par_read, s2_read, set ^ 1, 2 * i + 1);
                }
                if (kt_w >= 0 && i < 4) issue_w1(kt_w, i);
                if (kd_x >= 0) issue_x1(kd_x, i);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        auto stage_even = [&](int kt) {
            half(0, kt, 0, 1, -1, -1);          // multiply step 0, read step 1
            wait_lgkmcnt0();                    // stage kt is now fully in registers
            wait_vmcnt<16>();                   // my loads of stage kt+1 have landed
            __builtin_amdgcn_s_barrier();
            half(1, kt + 1, 1, 0, kt + 4, -1);  // multiply step 1, read step 0 of stage kt+1, refill W stage kt+4
        };
        auto stage_odd = [&](int kt) {
            half(0, kt, 1, 1, -1, -1);
            wait_lgkmcnt0();
            wait_vmcnt<4>();
            __builtin_amdgcn_s_barrier();
            half(1, kt + 1, 0, 0, kt + 4, (kt + 3) >> 1);   // also refill X stages kt+3, kt+4 (buffer of kt-1, kt)
        };

#pragma unroll
        for (int i = 0; i < 8; ++i) read_frag(0, 0, 0, 0, i);
        int kt = 0;
        for (; kt + 1 < KS; kt += 2) {
            stage_even(kt);
            stage_odd(kt + 1);
        }
        if (kt < KS) stage_even(kt);       // KS odd: one more even stage (its look-ahead reads are unused)
    } else {
        // fp8: a stage is 64 bytes = 64 values of K per row, exactly one v_mfma_f32_32x32x64_f8f6f4 per
        // accumulator (twice the flops per cycle of the K = 16 form).  A lane feeds the two 16-byte
        // chunks h and 2 + h of its weight column / activation row; the fragments of a whole stage
        // live in one of two register banks, the other bank is filled during the second half.
        typedef int v8i __attribute__((ext_vector_type(8)));
        v4i wq[2][2][4], xq[2][2][4];      // [bank][chunk 0/1][fragment]
        auto read_frag8 = [&](int kt, int kt_par, int bank, int i16) {
            const int s2 = i16 >> 3, i = i16 & 7;
            if (i < 4) {
                const int fn = i;
                const int blk = GATED ? (fn < 2 ? 2 * fn : 8 + 2 * (fn - 2)) : 2 * fn;
                wq[bank][s2][fn] = *reinterpret_cast<lds_v4i>(l3 + (kt & 3) * WBUF_BYTES + wf_off + blk * 1024 + s2 * 512);
            } else {
                const int fm = i - 4;
                xq[bank][s2][fm] = *reinterpret_cast<lds_v4i>(l3 + ((kt >> 1) & 1) * XBUF_BYTES + xf_off[2 * kt_par + s2] + fm * 4096);
            }
        };
        auto mma64 = [&](int bank, int fn, int fm) {
            const v8i a8 = __builtin_shufflevector(wq[bank][0][fn], wq[bank][1][fn], 0, 1, 2, 3, 4, 5, 6, 7);
            const v8i b8 = __builtin_shufflevector(xq[bank][0][fm], xq[bank][1][fm], 0, 1, 2, 3, 4, 5, 6, 7);
            acc[fn][fm] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, acc[fn][fm], 0, 0, 0, 0, 0, 0);
        };
        // PAR = kt & 1 = register bank of stage kt
        auto stage8 = [&](int kt, int par) {
#pragma unroll
            for (int i = 0; i < 8; ++i) mma64(par, i >> 2, i & 3);
            wait_lgkmcnt0();
            if (par) wait_vmcnt<4>(); else wait_vmcnt<16>();
            __builtin_amdgcn_s_barrier();
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                mma64(par, 2 + (i >> 2), i & 3);
                read_frag8(kt + 1, par ^ 1, par ^ 1, 2 * i);
                read_frag8(kt + 1, par ^ 1, par ^ 1, 2 * i + 1);
                if (i < 4) issue_w1(kt + 4, i);
                if (par) issue_x1((kt + 3) >> 1, i);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
#pragma unroll
        for (int i = 0; i < 16; ++i) read_frag8(0, 0, 0, i);
        int kt = 0;
        for (; kt + 1 < KS; kt += 2) {
            stage8(kt, 0);
            stage8(kt + 1, 1);
        }
        if (kt < KS) stage8(kt, 0);
    }
    wait_vmcnt<0>();
    __syncthreads();                       // every wave is done with the stage buffers
    advance();

    // Epilogue.  The 256 accumulators of a lane sit in the AGPR half of the register file: they can
    // be stored but not computed on there, and they cannot be indexed at run time.  So each wave
    // parks them in its own 32 KiB of the (now idle) LDS, 64 rows at a time, and reads them back
    // transposed, one quad (4 consecutive columns of one row) per lane: the QPR lanes that share a
    // row hold consecutive columns, so a store instruction writes whole 128-byte pieces of RPI rows
    // (quads stored from the MFMA layout would hit 32 rows per instruction, and the L2 takes such
    // fragments one request each).
    //   slot (fn, fmi, g) = 64 quads: rows fmi*32 + r32 of the 64, columns 8g + 4h .. +3 of fragment fn;
    //   the quad of lane L sits at position L ^ swz(fn, g, h), swz = ((fn%2)*4 + g)*2 + h, so the
    //   16 quads of a row that one quarter of a ds_read_b128 fetches fall into 16 different bank groups.
    // One wave per SIMD cannot overlap this with anybody's MFMAs, so what counts is the number of
    // vector instructions.  A whole tile (the common case) runs the loop fully unrolled: constant
    // LDS offsets, no bounds checks, one scalar pointer step per row group.  Ragged tiles run a
    // compact loop with the checks.
    v4f* stash = reinterpret_cast<v4f*>(lds) + wave * 2048;
    constexpr int QPR = GATED ? 16 : 32;            // output quads per row of this wave's part of the tile
    constexpr int RPI = 64 / QPR;                   // rows per iteration
    const int q = lane % QPR, rr = lane / QPR;
    const int fq = q >> 3, gq = (q >> 1) & 3, hq = q & 1;
    const int swz_q = ((fq & 1) * 4 + gq) * 2 + hq;
    const int nl = (GATED ? wn * 64 : wn * 128) + 4 * q;
    auto park = [&](int half) {
#pragma unroll
        for (int fn = 0; fn < 4; ++fn)
#pragma unroll
            for (int fmi = 0; fmi < 2; ++fmi)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    stash[((fn * 2 + fmi) * 4 + g) * 64 + (lane ^ (((fn & 1) * 4 + g) * 2 + h))] =
                        v4f{acc[fn][2 * half + fmi][4 * g], acc[fn][2 * half + fmi][4 * g + 1],
                            acc[fn][2 * half + fmi][4 * g + 2], acc[fn][2 * half + fmi][4 * g + 3]};
    };
    const bool vec_ok = (N & 3) == 0;
    if (vec_ok && rows == 256 && cols == (GATED ? 128 : 256)) {
        auto whole = [&](auto out_tag, auto tag) {
            constexpr int OUT = decltype(out_tag)::value, ACT = decltype(tag)::value;
            constexpr int OSZ = OUT == EPARA_BF16 ? 2 : 1;
            typedef float v2f __attribute__((ext_vector_type(2)));
            typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
            EPARA_GLOBAL char* ybase = as_global<char>(ga.Y) + (static_cast<size_t>(m0 + wm * 128) * N + n0) * OSZ;   // uniform
            const uint32_t lane_off = static_cast<uint32_t>((rr * N + nl) * OSZ);
            const int base_l = ((hq * 32) | rr) ^ swz_q;         // row & 31 = (it*RPI & 31) | rr, and | of disjoint bits = ^
            const float sg = ga.scale, su = ga.scale2 * ga.out_inv_scale, inv = ga.out_inv_scale;
            v4f b4 = {0.f, 0.f, 0.f, 0.f};
            if constexpr (!GATED) b4 = *reinterpret_cast<const __attribute__((address_space(3))) v4f*>(bias_tile + nl);
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                park(half);
#pragma unroll
                for (int it = 0; it < 64 / RPI; ++it) {
                    const int at = (base_l ^ ((it * RPI) & 31)) + gq * 64 + ((it * RPI) >> 5) * 256 + fq * 512;
                    float v[4];
                    if constexpr (GATED) {
                        const v4f gate = stash[at], up = stash[at + 1024];
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[i] = act_fast<EPARA_ACT_SILU>(sg * gate[i]) * (su * up[i]);
                    } else {
                        const v4f a4 = stash[at];
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[i] = act_fast<ACT>(sg * a4[i] + b4[i]) * inv;
                    }
                    EPARA_GLOBAL char* y = ybase + static_cast<size_t>(half * 64 + it * RPI) * N * OSZ + lane_off;
                    if constexpr (OUT == EPARA_BF16) {
                        v2u pk;
                        pk[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector((v2f{v[0], v[1]}), v2bf));
                        pk[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector((v2f{v[2], v[3]}), v2bf));
                        put<WT>(reinterpret_cast<EPARA_GLOBAL v2u*>(y), pk);
                    } else {
                        put<WT>(reinterpret_cast<EPARA_GLOBAL uint32_t*>(y), f32x4_to_e4m3(v[0], v[1], v[2], v[3]));
                    }
                }
            }
        };
        auto by_out = [&](auto tag) {
            if (DT == EPARA_BF16 || out_dtype == EPARA_BF16) whole(act_tag<EPARA_BF16>{}, tag);
            else if constexpr (DT != EPARA_BF16)              whole(act_tag<EPARA_FP8_E4M3>{}, tag);
        };
        if constexpr (GATED) by_out(act_tag<EPARA_ACT_SILU>{});
        else                 with_act(ga.act, by_out);
        return;
    }
    if constexpr (GATED) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            park(half);
#pragma unroll 2
            for (int it = 0; it < 64 / RPI; ++it) {
                const int row = it * RPI + rr, fmi = row >> 5;
                const int at = ((hq * 32 + (row & 31)) ^ swz_q) + gq * 64 + fmi * 256 + fq * 512;
                const v4f gate = stash[at], up = stash[at + 1024];
                finish_gated<WT>(ga, out_dtype, gate, up, m0, wm * 128 + half * 64 + row, rows, n0, nl, cols, vec_ok);
            }
        }
    } else {
        with_act(ga.act, [&](auto tag) {
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                park(half);
#pragma unroll 2
                for (int it = 0; it < 64 / RPI; ++it) {
                    const int row = it * RPI + rr, fmi = row >> 5;
                    const v4f a4 = stash[((hq * 32 + (row & 31)) ^ swz_q) + gq * 64 + fmi * 256 + fq * 512];
                    finish_plain<decltype(tag)::value, WT>(ga, out_dtype, a4, bias_tile, m0,
                                                       wm * 128 + half * 64 + row, rows, n0, nl, cols, vec_ok);
                }
            }
        });
    }
}

// ------------------------------------------------------------------ skinny tiles (weight streaming)

// Small batches are bandwidth bound: the weights are streamed from HBM exactly once, straight
// into MFMA operand registers (each load instruction of a wave reads 1 KiB of consecutive packed
// weights), while the activations are re-read from L2 by every tile, through a small LDS ring per
// wave (see skinny_setup).  To keep that re-read at half the weight traffic, a tile of streaming
// class c = 0, 1, 2 pairs MB = 1, 2, 4 blocks of 16 rows (the whole batch) with NFR = 2, 4, 8
// weight column blocks: 32 / 64 / 128 output columns, or for gated groups NFR/2 gate blocks and
// the matching NFR/2 up blocks (16 / 32 / 64 hidden columns).  K is walked in steps of two packed
// fragments (128 bytes of every activation row, so a row's cache line is used whole); wave w takes
// the steps p = w, w+4, ....  The four partial sums meet in LDS and are added in wave order: the
// result does not depend on timing.
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
    uint32_t xoff[8];      // per lane, per direct-load instruction j < 2 MB: byte offset of my row + my chunk's 16 c
    int KS, K;             // fragments along K, K
    int n_chunks;          // chunks of U steps per wave
};

// Activations of a step (two fragments = 128 bytes of K for MB x 16 rows) go through a per-wave LDS
// slot: direct-load instruction j covers rows 8j .. 8j+7 whole (8 x 128 bytes, eight cache lines),
// where loading MFMA operands straight from memory touches 16 half lines per instruction - the
// lines, not the bytes, are what the re-read of the activations costs next to the weight stream.
// Lane l of instruction j writes LDS chunk s = l%8 of row 8j + l/8 and fetches the global chunk
// c = s ^ ((row/2)%8); operand reads (16 rows x one chunk per quarter wave) then fall into 16
// different bank groups.
template <int DT, bool GATED, int MB, int NFR, int U>
__device__ __forceinline__ void skinny_setup(skinny_tile_state<NFR>& st, const epara_group_args& ga, int n0, int lane)
{
    constexpr int ESZ = DT == EPARA_BF16 ? 2 : 1;
    constexpr int EPC = 16 / ESZ, KF = 4 * EPC;
    const int K = ga.K, N = ga.N;
    const int KS = (K + KF - 1) / KF;
    const int NB = (N + 15) >> 4;
    st.K = K;
    st.KS = KS;
    const int steps = (KS + 1) >> 1;                             // two fragments per step
    st.n_chunks = (((steps + 3) >> 2) + U - 1) / U;
#pragma unroll
    for (int f = 0; f < NFR; ++f) {
        // gated: fragments 0 .. NFR/2-1 are gate blocks, the rest the same blocks of the up matrix
        const int rel = GATED ? (f % (NFR / 2)) : f;
        const int nb = min((n0 >> 4) + rel, NB - 1);             // a block past N only feeds unstored columns
        gcptr base = as_global<char>((GATED && f >= NFR / 2) ? ga.W2 : ga.W);
        st.w[f] = base + static_cast<size_t>(nb) * KS * 1024;
    }
    st.x = static_cast<const char*>(ga.X);
#pragma unroll
    for (int j = 0; j < 2 * MB; ++j) {
        const int row = 8 * j + (lane >> 3);
        const int c = (lane & 7) ^ ((row >> 1) & 7);
        st.xoff[j] = static_cast<uint32_t>(min(row, ga.M - 1)) * static_cast<uint32_t>(K * ESZ) + c * 16;
    }
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
    const int p = wave + 4 * i;                                  // step: fragments 2p and 2p+1
    // activations first: loads complete in issue order, so once the weights of this slot are in
    // their registers the slot's LDS image is complete too
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(st.x), 0, -1, 0x00020000);
    if ((2 * p + 2) * KF <= st.K) {                              // both fragments lie inside K
#pragma unroll
        for (int j = 0; j < 2 * MB; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xrsrc, (__attribute__((address_space(3))) void*)(xslot + j * 1024), 16,
                                                     static_cast<int>(st.xoff[j]), p * 128, 0, 0);
    } else {
        // ragged or padding step: a fragment past the last one repeats the last, a chunk past K
        // falls back to chunk 0 of its fragment (the packed weights are zero there)
#pragma unroll
        for (int j = 0; j < 2 * MB; ++j) {
            const int c = (lane & 7) ^ ((4 * j + (lane >> 4)) & 7);
            const int ks = min(2 * p + (c >> 2), st.KS - 1);
            const int cc = (ks * KF + (c & 3) * EPC < st.K) ? (c & 3) : 0;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xrsrc, (__attribute__((address_space(3))) void*)(xslot + j * 1024), 16,
                                                     static_cast<int>(st.xoff[j]) - c * 16 + ks * 64 + cc * 16, 0, 0, 0);
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
        if (2 * (wave + 4 * i) + e < st.KS) {
#pragma unroll
            for (int f = 0; f < NFR; ++f)
#pragma unroll
                for (int fm = 0; fm < MB; ++fm) mma<DT>(acc[f][fm], sl.w[e][f], x[e][fm]);
        }
    }
}

template <int DT, bool GATED, int MB, int NFR, bool WT>
__device__ __forceinline__ void skinny_finish(const epara_group_args& ga, int out_dtype, int n0, int cols,
                                              v4f (&acc)[NFR][MB], int wave, int lane, char* lds)
{
    const int r = lane & 15, q = lane >> 4;
    // red[wave][block of the pass][fm][lane]: at most 64 KiB, so the widest tile takes two passes
    constexpr int PASSES = (NFR * MB * 4096 + RING_LDS_OFFSET - 1) / RING_LDS_OFFSET;
    constexpr int NP = NFR / PASSES;                             // column blocks per pass
    v4f* red = reinterpret_cast<v4f*>(lds);
    const bool vec_ok = (ga.N & 3) == 0;
    const int M = ga.M;
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass) {
        __syncthreads();                                         // the previous sums have been read
#pragma unroll
        for (int fi = 0; fi < NP; ++fi) {
            // gated: a pass holds NP/2 gate blocks and the matching up blocks
            const int f = GATED ? (fi < NP / 2 ? pass * (NP / 2) + fi : NFR / 2 + pass * (NP / 2) + fi - NP / 2) : pass * NP + fi;
#pragma unroll
            for (int fm = 0; fm < MB; ++fm) red[((wave * NP + fi) * MB + fm) * 64 + lane] = acc[f][fm];
        }
        __syncthreads();
        if constexpr (GATED) {                                   // units (hidden column block p, row block fm)
            constexpr int UNITS = (NP / 2) * MB;
            for (int unit = wave; unit < UNITS; unit += 4) {
                const int pi = unit / MB, fm = unit % MB, p = pass * (NP / 2) + pi;
                if (fm * 16 >= M || p * 16 >= cols) continue;
                v4f g = {0.f, 0.f, 0.f, 0.f}, u = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    g += red[((w * NP + pi) * MB + fm) * 64 + lane];
                    u += red[((w * NP + NP / 2 + pi) * MB + fm) * 64 + lane];
                }
                finish_gated<WT>(ga, out_dtype, g, u, 0, fm * 16 + r, M, n0, p * 16 + 4 * q, cols, vec_ok);
            }
        } else {                                                 // units (column block f, row block fm)
            constexpr int UNITS = NP * MB;
            with_act(ga.act, [&](auto tag) {
                for (int unit = wave; unit < UNITS; unit += 4) {
                    const int fi = unit / MB, fm = unit % MB, f = pass * NP + fi;
                    if (fm * 16 >= M || f * 16 >= cols) continue;
                    v4f s0 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int w = 0; w < 4; ++w) s0 += red[((w * NP + fi) * MB + fm) * 64 + lane];
                    finish_plain<decltype(tag)::value, WT>(ga, out_dtype, s0, ga.bias ? as_global<float>(ga.bias) + n0 : nullptr, 0,
                                                       fm * 16 + r, M, n0, f * 16 + 4 * q, cols, vec_ok);
                }
            });
        }
    }
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
            if (c.pend_n[i] > 0)
                __hip_atomic_fetch_add(c.ws + CHAIN_HEADER_WORDS + c.counter_base + c.pend_group[i],
                                       static_cast<uint32_t>(c.pend_n[i]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t left = __hip_atomic_fetch_add(c.ws + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (left + 1 == gridDim.x) {
            for (int i = 0; i < n_counters; ++i)
                __hip_atomic_store(c.ws + CHAIN_HEADER_WORDS + i, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(c.ws + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Processes slot `slot` and every following slot of this workgroup that holds a tile of the same
// streaming class.  Returns the first slot it did not process.
template <int DT, bool GATED, bool CHAIN, int CLS, int MB, int NFR, int U>
__device__ __forceinline__ long skinny_run(const epara_group_args* __restrict__ args, const epara_tile* __restrict__ tiles,
                                           const int32_t* __restrict__ order, long slot, long n_slots, long stride,
                                           int out_dtype, char* lds, chain_ctx* chain)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    epara_tile tl = tiles[order[slot]];
    epara_group_args ga = args[tl.group];
    skinny_tile_state<NFR> cur, nxt;
    skinny_setup<DT, GATED, MB, NFR, U>(cur, ga, tl.n0, lane);
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
        int t_next = -1, stage = 0;
        bool have_next = false;
        epara_tile tl_next = tl;
        epara_group_args ga_next = ga;
        auto advance = [&]() {
            if (stage == 0)      { const long s1 = slot + stride; t_next = s1 < n_slots ? order[s1] : -1; }
            else if (stage == 1) { if (t_next >= 0) tl_next = tiles[t_next]; }
            else {
                have_next = t_next >= 0 && tl_next.cls == CLS;
                // in a chain the run ends before a tile that may have to wait for its input
                if constexpr (CHAIN) have_next = have_next && (tl_next.group == tl.group || !chain_must_wait(*chain, tl_next.group));
                if (have_next) ga_next = args[tl_next.group];
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
            skinny_setup<DT, GATED, MB, NFR, U>(nxt, ga_next, tl_next.n0, lane);
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
        skinny_finish<DT, GATED, MB, NFR, CHAIN>(ga, out_dtype, tl.n0, tl.cols, acc, wave, lane, lds);
        if constexpr (CHAIN) chain_done(*chain, tl.group);
        if (slot_next < 0) break;
        slot = slot_next;
        tl = tl_next;
        ga = ga_next;
        cur = nxt;
    }
    // first slot after this run: the next non-idle slot of this workgroup or the end
    for (slot += stride; slot < n_slots && order[slot] < 0; slot += stride) {}
    return slot;
}

// ------------------------------------------------------------------ persistent kernels

constexpr int N_STREAM_CLASSES = 3;

// Streaming classes: (row blocks, weight column blocks, ring depth) = (1, 2, 4), (2, 4, 3) and
// (4, 8, 2) or, in a launch planned with the narrow table, (4, 4, 3).
template <int DT, bool GATED, bool CHAIN = false>
__device__ __forceinline__ void grouped_body(const epara_group_args* __restrict__ args, const epara_tile* __restrict__ tiles,
                                             const int32_t* __restrict__ order, long n_slots, int out_dtype, int narrow, char* lds,
                                             chain_ctx* chain = nullptr)
{
    const long stride = gridDim.x;
    long s = blockIdx.x;
    while (s < n_slots) {
        const int t = order[s];
        if (t < 0) { s += stride; continue; }
        const epara_tile tl = tiles[t];
        if constexpr (CHAIN) chain_wait(*chain, tl.group);
        if (tl.cls == 0)      s = skinny_run<DT, GATED, CHAIN, 0, 1, 2, 4>(args, tiles, order, s, n_slots, stride, out_dtype, lds, chain);
        else if (tl.cls == 1) s = skinny_run<DT, GATED, CHAIN, 1, 2, 4, 3>(args, tiles, order, s, n_slots, stride, out_dtype, lds, chain);
        else if (tl.cls == 2 && !narrow) s = skinny_run<DT, GATED, CHAIN, 2, 4, 8, 2>(args, tiles, order, s, n_slots, stride, out_dtype, lds, chain);
        else if (tl.cls == 2) s = skinny_run<DT, GATED, CHAIN, 2, 4, 4, 3>(args, tiles, order, s, n_slots, stride, out_dtype, lds, chain);
        else {
            // A run of panel tiles.  What follows a tile in the workgroup's list is found by three
            // dependent scalar loads (order -> tile -> group arguments); they are issued one at a time
            // from inside the tile before, so the next tile starts without waiting for them.
            epara_tile cur = tl;
            epara_group_args ga = args[cur.group];
            for (;;) {
                if constexpr (CHAIN) chain_wait(*chain, cur.group);
                const long s1 = s + stride;
                int t1 = -1, stage = 0;
                epara_tile nxt = cur;
                epara_group_args ga1 = ga;
                auto advance = [&]() {
                    if (stage == 0)      { t1 = s1 < n_slots ? order[s1] : -1; }
                    else if (stage == 1) { if (t1 >= 0) nxt = tiles[t1]; }
                    else                 { if (t1 >= 0 && nxt.cls >= N_STREAM_CLASSES) ga1 = args[nxt.group]; }
                    ++stage;
                };
                big_tile<DT, GATED, CHAIN>(ga, out_dtype, cur.m0, cur.n0, cur.rows, cur.cols, lds, advance);
                if constexpr (CHAIN) chain_done(*chain, cur.group);
                s = s1;
                if (t1 < 0 || nxt.cls < N_STREAM_CLASSES) break;   // idle slot, end of the list or a streaming tile
                cur = nxt;
                ga = ga1;
            }
        }
    }
}

template <int DT>
__global__ __launch_bounds__(NT) void grouped_kernel(const epara_group_args* __restrict__ args,
                                                     const epara_tile* __restrict__ tiles,
                                                     const int32_t* __restrict__ order,
                                                     long n_slots, int out_dtype, int gated, int narrow)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    if (gated) grouped_body<DT, true>(args, tiles, order, n_slots, out_dtype, narrow, lds);
    else       grouped_body<DT, false>(args, tiles, order, n_slots, out_dtype, narrow, lds);
}

// fp32 groups of at most 16 rows: a 16 x 64 tile with K cut into four contiguous quarters, one per
// wave (a tile of a small model is a chain of dependent memory latencies, and this chain is four
// times shorter).  Each wave stages its 16 x F32S_BK activations and F32S_BK x 64 weights in its own
// part of the LDS (no barrier inside the K loop: a wave's LDS operations run in order), a lane
// holds 4 rows x 4 columns; the four partial tiles are then added in wave order 0, 1, 2, 3, so the
// result depends on nothing but the operands.
constexpr int F32S_BM = 16, F32S_BN = 64, F32S_BK = 16;

template <bool CHAIN>
__device__ __forceinline__ void f32_small_tile(const epara_group_args& ga, const epara_tile& tl)
{
    __shared__ float Xq[4][F32S_BK][F32S_BM + 1];
    __shared__ float Wq[4][F32S_BK][F32S_BN];
    __shared__ float part[4][F32S_BM][F32S_BN];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tx = lane & 15, ty = lane >> 4;
    const EPARA_GLOBAL float* X = as_global<float>(ga.X);
    const EPARA_GLOBAL float* W = as_global<float>(ga.W);
    const int K = ga.K, N = ga.N;
    const int Kq = (K + 3) / 4;
    const int k_begin = wave * Kq, k_end = min(K, k_begin + Kq);
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    float xr[4], wr[16];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {                       // X: element e = lane + 64 j -> row e / 16, k e % 16
            const int e = lane + 64 * j, row = e >> 4, kk = e & 15;
            xr[j] = (row < tl.rows && k0 + kk < k_end) ? X[static_cast<size_t>(tl.m0 + row) * K + k0 + kk] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 16; ++j)                        // W: row k0 + j, column lane
            wr[j] = (k0 + j < k_end && lane < tl.cols) ? W[static_cast<size_t>(k0 + j) * N + tl.n0 + lane] : 0.f;
    };
    fetch(k_begin);
    for (int k0 = k_begin; k0 < k_end; k0 += F32S_BK) {
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = lane + 64 * j;
            Xq[wave][e & 15][e >> 4] = xr[j];
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) Wq[wave][j][lane] = wr[j];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (k0 + F32S_BK < k_end) fetch(k0 + F32S_BK);
#pragma unroll
        for (int kk = 0; kk < F32S_BK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = Xq[wave][kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Wq[wave][kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) part[wave][ty * 4 + i][tx * 4 + j] = acc[i][j];
    __syncthreads();
    {
        const int row = tid >> 4, c0 = (tid & 15) * 4;      // 16 rows x 16 column quads over 256 threads
        EPARA_GLOBAL float* Y = as_global<float>(ga.Y);
        with_act(ga.act, [&](auto tag) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = c0 + j;
                if (row >= tl.rows || col >= tl.cols) continue;
                const float sum = ((part[0][row][col] + part[1][row][col]) + part[2][row][col]) + part[3][row][col];
                const float b = ga.bias ? as_global<float>(ga.bias)[tl.n0 + col] : 0.f;
                put<CHAIN>(Y + static_cast<size_t>(tl.m0 + row) * N + tl.n0 + col,
                           act_apply<decltype(tag)::value>(ga.scale * sum + b));
            }
        });
    }
    __syncthreads();                                        // the partial tiles are free again
}

// fp32 groups: batches of more than 16 rows in 64x64 tiles, plain FMA in fp32, K ascending; smaller
// batches in f32_small_tile.
template <bool CHAIN>
__device__ __forceinline__ void f32_body(const epara_group_args* __restrict__ args, const epara_tile* __restrict__ tiles,
                                         const int32_t* __restrict__ order, long n_slots, chain_ctx* chain)
{
    __shared__ float Xs[F32_BK][F32_BM + 1];
    __shared__ float Ws[F32_BK][F32_BN];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    for (long s = blockIdx.x; s < n_slots; s += gridDim.x) {
        const int t = order[s];
        if (t < 0) continue;
        const epara_tile tl = tiles[t];
        if constexpr (CHAIN) chain_wait(*chain, tl.group);
        const epara_group_args ga = args[tl.group];
        if (tl.cls == 0) {                                  // class 0 of the fp32 table: at most 16 rows
            f32_small_tile<CHAIN>(ga, tl);
            if constexpr (CHAIN) chain_done(*chain, tl.group);
            continue;
        }
        const EPARA_GLOBAL float* X = as_global<float>(ga.X);
        const EPARA_GLOBAL float* W = as_global<float>(ga.W);
        EPARA_GLOBAL float* Y = as_global<float>(ga.Y);
        const int K = ga.K, N = ga.N;
        float acc[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
        // The K steps are software pipelined through registers: the loads of step k0 + BK are in flight
        // while step k0 is multiplied (a tile of a small model is a chain of dependent memory
        // latencies otherwise).  The sums still run over K in ascending order.
        float xr[F32_PER], wr[F32_PER];
        auto fetch = [&](int k0) {
#pragma unroll
            for (int j = 0; j < F32_PER; ++j) {
                const int e = tid + F32_NT * j;
                const int row = e / F32_BK, kk = e % F32_BK;
                xr[j] = (row < tl.rows && k0 + kk < K) ? X[static_cast<size_t>(tl.m0 + row) * K + k0 + kk] : 0.f;
                const int kw = e >> 6, nn = e & 63;
                wr[j] = (k0 + kw < K && nn < tl.cols) ? W[static_cast<size_t>(k0 + kw) * N + tl.n0 + nn] : 0.f;
            }
        };
        fetch(0);
        for (int k0 = 0; k0 < K; k0 += F32_BK) {
            __syncthreads();
#pragma unroll
            for (int j = 0; j < F32_PER; ++j) {
                const int e = tid + F32_NT * j;
                Xs[e % F32_BK][e / F32_BK] = xr[j];
                Ws[e >> 6][e & 63] = wr[j];
            }
            __syncthreads();
            if (k0 + F32_BK < K) fetch(k0 + F32_BK);
#pragma unroll
            for (int kk = 0; kk < F32_BK; ++kk) {
                float a[4], b[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) a[i] = Xs[kk][ty * 4 + i];
#pragma unroll
                for (int j = 0; j < 4; ++j) b[j] = Ws[kk][tx * 4 + j];
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
            }
        }
        with_act(ga.act, [&](auto tag) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = ty * 4 + i;
                if (row >= tl.rows) continue;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int col = tx * 4 + j;
                    if (col >= tl.cols) continue;
                    const float b = ga.bias ? as_global<float>(ga.bias)[tl.n0 + col] : 0.f;
                    put<CHAIN>(Y + static_cast<size_t>(tl.m0 + row) * N + tl.n0 + col,
                               act_apply<decltype(tag)::value>(ga.scale * acc[i][j] + b));
                }
            }
        });
        if constexpr (CHAIN) chain_done(*chain, tl.group);
    }
}

__global__ __launch_bounds__(F32_NT) void grouped_kernel_f32(const epara_group_args* __restrict__ args,
                                                             const epara_tile* __restrict__ tiles,
                                                             const int32_t* __restrict__ order, long n_slots)
{
    f32_body<false>(args, tiles, order, n_slots, nullptr);
}

// ---- a chain of launches as one kernel: the phases one after the other in every workgroup
//
// The tables of every phase are kernel arguments of their own (not fields of a structure in memory):
// only then does the compiler know them as read-only global memory that nothing in the kernel
// writes, and fetch tile, order and argument records with scalar loads as in the single-launch
// kernel -- the streaming pipeline counts its outstanding vector loads and has no room for others.
struct chain_scalars {
    long n_slots[EPARA_MAX_CHAIN_PHASES];
    int out_dtype[EPARA_MAX_CHAIN_PHASES], narrow[EPARA_MAX_CHAIN_PHASES], counter_base[EPARA_MAX_CHAIN_PHASES];
    uint32_t* ws;
    uint32_t spin_limit;
    int n_phases, n_counters;
};

#define CHAIN_TABLES(i) const epara_group_args* __restrict__ a##i, const epara_tile* __restrict__ t##i, \
                        const int32_t* __restrict__ o##i, const epara_chain_wait* __restrict__ w##i
#define CHAIN_PICK(p, x) ((p) == 0 ? x##0 : (p) == 1 ? x##1 : (p) == 2 ? x##2 : x##3)

__device__ __forceinline__ chain_ctx chain_begin(const chain_scalars& S)
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
                                                           const chain_scalars S)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    chain_ctx c = chain_begin(S);
    if constexpr (FFN) {
        chain_enter_phase(c, nullptr, S.counter_base[0]);
        grouped_body<DT, true, true>(a0, t0, o0, S.n_slots[0], S.out_dtype[0], S.narrow[0], lds, &c);
        chain_enter_phase(c, w1, S.counter_base[1]);
        grouped_body<DT, false, true>(a1, t1, o1, S.n_slots[1], S.out_dtype[1], S.narrow[1], lds, &c);
    } else {
        for (int p = 0; p < S.n_phases; ++p) {
            chain_enter_phase(c, CHAIN_PICK(p, w), S.counter_base[p]);
            grouped_body<DT, false, true>(CHAIN_PICK(p, a), CHAIN_PICK(p, t), CHAIN_PICK(p, o), S.n_slots[p], S.out_dtype[p],
                                          S.narrow[p], lds, &c);
        }
    }
    chain_exit(c, S.n_counters);
}

__global__ __launch_bounds__(F32_NT) void grouped_chain_kernel_f32(CHAIN_TABLES(0), CHAIN_TABLES(1), CHAIN_TABLES(2), CHAIN_TABLES(3),
                                                                   const chain_scalars S)
{
    chain_ctx c = chain_begin(S);
    for (int p = 0; p < S.n_phases; ++p) {
        chain_enter_phase(c, CHAIN_PICK(p, w), S.counter_base[p]);
        f32_body<true>(CHAIN_PICK(p, a), CHAIN_PICK(p, t), CHAIN_PICK(p, o), S.n_slots[p], &c);
    }
    chain_exit(c, S.n_counters);
}

__global__ void fill_words_kernel(uint32_t* p, long n, uint32_t v)
{
    for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += static_cast<long>(gridDim.x) * blockDim.x) p[i] = v;
}

// One 16-byte chunk of the packed weights per thread.
template <int ESZ>
__global__ void pack_kernel(const char* __restrict__ W, int K, int N, char* __restrict__ out, long n_chunks)
{
    constexpr int EPC = 16 / ESZ, KF = 4 * EPC;
    const long idx = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (idx >= n_chunks) return;
    const int KS = (K + KF - 1) / KF;
    const int slot = static_cast<int>(idx & 63);
    const long frag = idx >> 6;
    const int ks = static_cast<int>(frag % KS);
    const long nb = frag / KS;
    const int q = slot >> 4, r = slot & 15;
    const long n = nb * 16 + r;
    const int k0 = ks * KF + q * EPC;
    alignas(16) char buf[16];
#pragma unroll
    for (int e = 0; e < EPC; ++e) {
        const int k = k0 + e;
        const bool ok = k < K && n < N;
        if constexpr (ESZ == 2) {
            reinterpret_cast<uint16_t*>(buf)[e] = ok ? reinterpret_cast<const uint16_t*>(W)[static_cast<size_t>(k) * N + n] : 0;
        } else {
            reinterpret_cast<uint8_t*>(buf)[e] = ok ? reinterpret_cast<const uint8_t*>(W)[static_cast<size_t>(k) * N + n] : 0;
        }
    }
    *reinterpret_cast<v4i*>(out + idx * 16) = *reinterpret_cast<const v4i*>(buf);
}

// ------------------------------------------------------------------ host-side validation

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

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
    int32_t last = EPARA_OK;
    for (int narrow = 0; narrow < (f32 ? 1 : 2); ++narrow) {
        last = check_tiles(L, in_dtype, narrow);
        if (last == EPARA_OK) { if (narrow_out) *narrow_out = narrow; return EPARA_OK; }
    }
    return last;
}

int32_t enqueue(const epara_launch* L, int32_t in_dtype, int32_t out_dtype, int narrow, hipStream_t stream)
{
    if (L->n_tiles == 0) return EPARA_OK;
    int gated = 0;
    for (int32_t g = 0; g < L->G; ++g)
        if (L->h_args[g].M > 0 && L->h_args[g].act == EPARA_ACT_SWIGLU) gated = 1;
    const dim3 grid(static_cast<unsigned>(L->n_workgroups));
    (void)hipGetLastError();
    if (in_dtype == EPARA_F32) {
        hipLaunchKernelGGL(grouped_kernel_f32, grid, dim3(F32_NT), 0, stream, L->d_args, L->d_tiles, L->d_order,
                           static_cast<long>(L->n_slots));
    } else if (in_dtype == EPARA_BF16) {
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&grouped_kernel<EPARA_BF16>),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (attr != hipSuccess) return EPARA_ERR_HIP;
        hipLaunchKernelGGL(grouped_kernel<EPARA_BF16>, grid, dim3(NT), LDS_BYTES, stream, L->d_args, L->d_tiles,
                           L->d_order, static_cast<long>(L->n_slots), out_dtype, gated, narrow);
    } else {
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&grouped_kernel<EPARA_FP8_E4M3>),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (attr != hipSuccess) return EPARA_ERR_HIP;
        hipLaunchKernelGGL(grouped_kernel<EPARA_FP8_E4M3>, grid, dim3(NT), LDS_BYTES, stream, L->d_args, L->d_tiles,
                           L->d_order, static_cast<long>(L->n_slots), out_dtype, gated, narrow);
    }
    return hipGetLastError() == hipSuccess ? EPARA_OK : EPARA_ERR_HIP;
}

}  // namespace

extern "C" {

int64_t epara_packed_weight_bytes(int32_t K, int32_t N, int32_t dtype)
{
    if (K <= 0 || N <= 0) return -1;
    if (dtype == EPARA_F32) return static_cast<int64_t>(K) * N * 4;
    if (dtype != EPARA_BF16 && dtype != EPARA_FP8_E4M3) return -1;
    const int64_t KF = dtype == EPARA_BF16 ? 32 : 64;
    return ((static_cast<int64_t>(N) + 15) / 16) * ((K + KF - 1) / KF) * 1024;
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
    const long n_chunks = need / 16;
    const unsigned blocks = static_cast<unsigned>((n_chunks + 255) / 256);
    if (dtype == EPARA_BF16)
        hipLaunchKernelGGL(pack_kernel<2>, dim3(blocks), dim3(256), 0, st, static_cast<const char*>(d_W), K, N,
                           static_cast<char*>(d_packed), n_chunks);
    else
        hipLaunchKernelGGL(pack_kernel<1>, dim3(blocks), dim3(256), 0, st, static_cast<const char*>(d_W), K, N,
                           static_cast<char*>(d_packed), n_chunks);
    return hipGetLastError() == hipSuccess ? EPARA_OK : EPARA_ERR_HIP;
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
    const long n = bytes / 4;
    hipLaunchKernelGGL(fill_words_kernel, dim3(static_cast<unsigned>(n < 65536 ? (n + 255) / 256 : 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<uint32_t*>(d_workspace), n, 0u);
    return hipGetLastError() == hipSuccess ? EPARA_OK : EPARA_ERR_HIP;
}

int32_t epara_grouped_chain(const epara_chain_phase* phases, int32_t n_phases, int32_t in_dtype,
                            void* d_workspace, int64_t workspace_bytes, uint32_t spin_limit, void* stream)
{
    if (!phases || !d_workspace) return EPARA_ERR_NULL;
    if (n_phases < 1 || n_phases > EPARA_MAX_CHAIN_PHASES) return EPARA_ERR_SHAPE;
    if (!aligned16(d_workspace)) return EPARA_ERR_ALIGN;
    chain_scalars S;
    std::memset(&S, 0, sizeof S);
    const epara_group_args* d_args[EPARA_MAX_CHAIN_PHASES] = {};
    const epara_tile* d_tiles[EPARA_MAX_CHAIN_PHASES] = {};
    const int32_t* d_order[EPARA_MAX_CHAIN_PHASES] = {};
    const epara_chain_wait* d_waits[EPARA_MAX_CHAIN_PHASES] = {};
    int gated[EPARA_MAX_CHAIN_PHASES] = {};
    int32_t n_counters = 0, n_workgroups = 0;
    bool any = false;
    for (int32_t p = 0; p < n_phases; ++p) {
        const epara_chain_phase& ph = phases[p];
        const epara_launch* L = ph.launch;
        int narrow = 0;
        if (int32_t st = validate_launch(L, in_dtype, ph.out_dtype, &narrow)) return st;
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
            }
            d_waits[p] = ph.d_waits;
        }
        d_args[p] = L->d_args; d_tiles[p] = L->d_tiles; d_order[p] = L->d_order;
        S.n_slots[p] = L->n_tiles > 0 ? L->n_slots : 0;
        S.out_dtype[p] = ph.out_dtype; S.narrow[p] = narrow; S.counter_base[p] = ph.counter_base;
    }
    // the kernels exist for chains without gating and for the two phases of a SwiGLU FFN
    bool ffn = false;
    for (int32_t p = 0; p < n_phases; ++p) ffn = ffn || gated[p];
    if (ffn && !(n_phases == 2 && gated[0] && !gated[1])) return EPARA_ERR_DTYPE;
    if (workspace_bytes < epara_chain_workspace_bytes(n_counters)) return EPARA_ERR_CAPACITY;
    if (!any) return EPARA_OK;
    S.ws = static_cast<uint32_t*>(d_workspace);
    S.spin_limit = spin_limit ? spin_limit : (1u << 20);
    S.n_phases = n_phases;
    S.n_counters = n_counters;

    hipStream_t st = static_cast<hipStream_t>(stream);
    typedef void (*kernel_t)(const epara_group_args*, const epara_tile*, const int32_t*, const epara_chain_wait*,
                             const epara_group_args*, const epara_tile*, const int32_t*, const epara_chain_wait*,
                             const epara_group_args*, const epara_tile*, const int32_t*, const epara_chain_wait*,
                             const epara_group_args*, const epara_tile*, const int32_t*, const epara_chain_wait*, chain_scalars);
    kernel_t fn = in_dtype == EPARA_F32 ? grouped_chain_kernel_f32
                : in_dtype == EPARA_BF16 ? (ffn ? grouped_chain_kernel<EPARA_BF16, true> : grouped_chain_kernel<EPARA_BF16, false>)
                                         : (ffn ? grouped_chain_kernel<EPARA_FP8_E4M3, true> : grouped_chain_kernel<EPARA_FP8_E4M3, false>);
    const int threads = in_dtype == EPARA_F32 ? F32_NT : NT;
    const size_t dyn = in_dtype == EPARA_F32 ? 0 : LDS_BYTES;
    (void)hipGetLastError();
    // a waiting workgroup must not keep the one it waits for off the GPU: the whole grid has to be resident
    struct limit { int dev; const void* fn; int64_t resident; };
    static thread_local limit cache[8] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return EPARA_ERR_HIP;
    int64_t resident = -1;
    for (const limit& l : cache)
        if (l.fn == reinterpret_cast<const void*>(fn) && l.dev == dev) resident = l.resident;
    if (resident < 0) {
        int per_cu = 0, cus = 0;
        if (dyn && hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess)
            return EPARA_ERR_HIP;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(fn), threads, dyn) != hipSuccess) return EPARA_ERR_HIP;
        resident = static_cast<int64_t>(per_cu) * cus;
        static thread_local int next = 0;
        cache[next++ % 8] = {dev, reinterpret_cast<const void*>(fn), resident};
    }
    if (static_cast<int64_t>(n_workgroups) > resident) return EPARA_ERR_SHAPE;
    hipLaunchKernelGGL(fn, dim3(static_cast<unsigned>(n_workgroups)), dim3(threads), dyn, st,
                       d_args[0], d_tiles[0], d_order[0], d_waits[0], d_args[1], d_tiles[1], d_order[1], d_waits[1],
                       d_args[2], d_tiles[2], d_order[2], d_waits[2], d_args[3], d_tiles[3], d_order[3], d_waits[3], S);
    return hipGetLastError() == hipSuccess ? EPARA_OK : EPARA_ERR_HIP;
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
