// libepara: what lies between the dense layers of a vision-transformer encoder block (the ViT services of
// the paper's co-located setting, Sec. 3.1 MT): residual + layer normalisation, and attention.
//
//   epara_add_layernorm   s = x + r, y = LN(s) * gamma + beta, a wave per row        (bound by HBM traffic)
//   epara_attention       softmax(Q K^T / sqrt(d_h)) V per image and head, MFMA 16x16x32 bf16
//
// Attention at ViT sizes (197 tokens, d_h = 64) is small: a head's keys and values are 25 KB each, so a
// workgroup holds them in the LDS and forms every score of a block of 16 queries at once: no running maximum,
// no rescaling.  Both matrix products are written "transposed" so that a lane's accumulator quad already is
// the next operand:
//   S^T = K Q^T   A = 16 keys x 32 dims (LDS), B = 32 dims x 16 queries (registers, from global memory);
//                 lane (j = lane % 16, g = lane / 16) then holds the scores of query j against keys
//                 4 g .. 4 g + 3 of every block of 16 keys: a row of S is spread over the four lanes
//                 j, j + 16, j + 32, j + 48 and their registers (max and sum: registers, then two shuffles);
//   O^T = V^T P^T A = 16 dims x 32 keys (LDS, values stored transposed), B = 32 keys x 16 queries = the
//                 exponentials of two key blocks, packed to bf16 in place.  Only the pairing of A and B
//                 along the contraction matters, so "key slot 8 g + e" means key 4 g + e of the first block
//                 (e < 4) or key 4 g + e - 4 of the second in both operands.  The same freedom orders the rows of
//                 V^T so that a lane ends with 16 consecutive output columns of its query: two 16-byte stores.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "epara.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
#define EPARA_GLOBAL __attribute__((address_space(1)))

constexpr int NT = 256;
constexpr int NORM_GRID = 1024;          // workgroups of the normalisation kernel: four per compute unit, a few rows per wave

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
// two fp32 -> two bf16 (round to nearest even, in hardware), low half first
__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((v2f{a, b}), v2bf));
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
    return v;
}

// ---- residual + layer normalisation ---------------------------------------------------------------------

// Group of row `row`: the last one whose first_row is <= row (groups without rows are skipped by the rule itself).
__device__ __forceinline__ int find_norm_group(const epara_norm_args* __restrict__ args, int G, int row)
{
    int lo = 0, hi = G - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (args[mid].first_row <= row) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// A row on its way through a wave: CH 16-byte chunks (8 values) per lane, lane l holds chunks l, l + 64, ... of it.
template <int CH>
struct norm_row_regs {
    epara_norm_args a;     // the row's group (the same for all lanes)
    int row;               // its index inside the group
    v4i x[CH], r[CH];
};

template <int CH>
__device__ __forceinline__ void norm_load(const epara_norm_args* __restrict__ args, int G, int global_row, int lane, norm_row_regs<CH>& q)
{
    q.a = args[find_norm_group(args, G, global_row)];
    q.row = global_row - q.a.first_row;
    const int n_chunks = q.a.d >> 3;
    const size_t base = static_cast<size_t>(q.row) * q.a.d * 2;
    const EPARA_GLOBAL char* x = (const EPARA_GLOBAL char*)q.a.X + base;
    const EPARA_GLOBAL char* r = q.a.R ? (const EPARA_GLOBAL char*)q.a.R + base : nullptr;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int chunk = c * 64 + lane;
        q.x[c] = v4i{0, 0, 0, 0};
        q.r[c] = v4i{0, 0, 0, 0};
        if (chunk < n_chunks) {
            q.x[c] = *reinterpret_cast<const EPARA_GLOBAL v4i*>(x + chunk * 16);
            if (r) q.r[c] = *reinterpret_cast<const EPARA_GLOBAL v4i*>(r + chunk * 16);
        }
    }
}

template <int CH>
__device__ __forceinline__ void norm_finish(const norm_row_regs<CH>& q, int lane)
{
    const epara_norm_args& a = q.a;
    const int d = a.d, n_chunks = d >> 3;
    const size_t base = static_cast<size_t>(q.row) * d * 2;
    // scale and shift of my columns: asked for before the reductions, so that they arrive under them
    const EPARA_GLOBAL float* gamma = (const EPARA_GLOBAL float*)a.gamma;
    const EPARA_GLOBAL float* beta = (const EPARA_GLOBAL float*)a.beta;
    constexpr bool EARLY = CH <= 4;                       // wide rows have no registers to spare for it
    v4f gm[EARLY ? CH : 1][2], bt[EARLY ? CH : 1][2];
    auto scale_shift = [&](int c, int chunk) {
        gm[c][0] = *reinterpret_cast<const EPARA_GLOBAL v4f*>(gamma + chunk * 8);
        gm[c][1] = *reinterpret_cast<const EPARA_GLOBAL v4f*>(gamma + chunk * 8 + 4);
        bt[c][0] = *reinterpret_cast<const EPARA_GLOBAL v4f*>(beta + chunk * 8);
        bt[c][1] = *reinterpret_cast<const EPARA_GLOBAL v4f*>(beta + chunk * 8 + 4);
    };
    if constexpr (EARLY) {
#pragma unroll
        for (int c = 0; c < CH; ++c)
            if (c * 64 + lane < n_chunks) scale_shift(c, c * 64 + lane);
    }
    float s[CH][8];
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t xu = static_cast<uint32_t>(q.x[c][j]), ru = static_cast<uint32_t>(q.r[c][j]);
            s[c][2 * j] = bf16_lo(xu) + bf16_lo(ru);          // chunks past the row hold zeros and add nothing
            s[c][2 * j + 1] = bf16_hi(xu) + bf16_hi(ru);
            sum += s[c][2 * j] + s[c][2 * j + 1];
        }
    const float fd = static_cast<float>(d);
    const float mu = wave_sum(sum) / fd;                  // a division: a constant row gives exactly its value, and y = beta
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c)
        if (c * 64 + lane < n_chunks) {
#pragma unroll
            for (int j = 0; j < 8; ++j) { const float t = s[c][j] - mu; sq += t * t; }
        }
    const float var = wave_sum(sq) / fd;
    const float rstd = 1.f / sqrtf(var + a.eps);
    EPARA_GLOBAL char* so = a.S ? (EPARA_GLOBAL char*)a.S + base : nullptr;
    EPARA_GLOBAL char* yo = (EPARA_GLOBAL char*)a.Y + base;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int chunk = c * 64 + lane;
        if (chunk >= n_chunks) continue;
        const int gc = EARLY ? c : 0;
        if constexpr (!EARLY) scale_shift(0, chunk);
        float y[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            y[j] = (s[c][j] - mu) * rstd * gm[gc][0][j] + bt[gc][0][j];
            y[4 + j] = (s[c][4 + j] - mu) * rstd * gm[gc][1][j] + bt[gc][1][j];
        }
        v4i out;
        if (so) {
#pragma unroll
            for (int j = 0; j < 4; ++j) out[j] = static_cast<int>(pack_bf16(s[c][2 * j], s[c][2 * j + 1]));
            *reinterpret_cast<EPARA_GLOBAL v4i*>(so + chunk * 16) = out;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) out[j] = static_cast<int>(pack_bf16(y[2 * j], y[2 * j + 1]));
        *reinterpret_cast<EPARA_GLOBAL v4i*>(yo + chunk * 16) = out;
    }
}

// A wave walks rows wave, wave + (waves of the grid), ... and (narrow rows) has the loads of its next row in flight
// while it reduces and stores the current one.  CH = chunks per lane that the widest group of the launch needs (narrower rows
// leave chunks empty): one kernel per CH, so that the common narrow rows do not pay for the registers of the widest.
template <int CH>
__global__ __launch_bounds__(NT) void add_layernorm_kernel(const epara_norm_args* __restrict__ args, int G, int n_rows)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int stride = gridDim.x * (NT / 64);
    int row = blockIdx.x * (NT / 64) + wave;
    if (row >= n_rows) return;
    if constexpr (CH <= 4) {
        norm_row_regs<CH> cur, nxt;
        norm_load<CH>(args, G, row, lane, cur);
        for (;;) {
            const int next = row + stride;
            const bool more = next < n_rows;
            if (more) norm_load<CH>(args, G, next, lane, nxt);
            norm_finish<CH>(cur, lane);
            if (!more) break;
            cur = nxt;
            row = next;
        }
    } else {                                              // a wide row alone is 8 KiB or more of loads in flight
        for (; row < n_rows; row += stride) {
            norm_row_regs<CH> cur;
            norm_load<CH>(args, G, row, lane, cur);
            norm_finish<CH>(cur, lane);
        }
    }
}

// ---- attention --------------------------------------------------------------------------------------------

constexpr int DH = EPARA_ATTN_HEAD_DIM;                   // 64: two MFMA steps of 32 along the head dimension
constexpr int MAX_KB = EPARA_ATTN_MAX_TOKENS / 16;        // key blocks of 16
constexpr int K_ROW = DH * 2;                             // bytes of a key row in the LDS: 8 chunks of 16, chunk c at c ^ (key % 8)
static_assert(MAX_KB % 2 == 0, "the second product takes key blocks in pairs");
constexpr int NT_ATTN = 512, ATTN_WAVES = NT_ATTN / 64;  // eight waves share a head's keys and values: two or one query block each at ViT sizes

// Group of item `item`: the last one whose first_item is <= item.  Up to 64 groups: every lane looks at one group
// and the wave counts (one memory latency); more: bisection.
__device__ __forceinline__ int find_attn_group(const epara_attn_args* __restrict__ args, int G, int item, int lane)
{
    if (G <= 64) {
        const int first = lane < G ? args[lane].first_item : 0x7fffffff;
        return __builtin_popcountll(__ballot(first <= item)) - 1;        // first_item never decreases, group 0 starts at 0
    }
    int lo = 0, hi = G - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (args[mid].first_item <= item) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// KB = key blocks of 16 that the kernel multiplies for every image (even; the host takes the smallest instance that
// holds the longest image of the launch): the loops over key blocks have no conditions in them, so the LDS reads
// of a block run ahead of the products of the one before.  Keys past an image are zero rows whose scores are masked.
template <int KB>
__global__ __launch_bounds__(NT_ATTN, 4) void attention_kernel(const epara_attn_args* __restrict__ args, int G)
{
    constexpr int KEYS = KB * 16;
    constexpr int VT_ROW = KEYS * 2 + 8;                  // bytes of a row of V^T (one head dimension, all keys) + 8: rows fall on different banks
    constexpr int MAX_QB = (KB + ATTN_WAVES - 1) / ATTN_WAVES;                       // query blocks of 16 per wave
    constexpr int STAGE_STEPS = (KEYS / 2 * 8 + NT_ATTN - 1) / NT_ATTN;              // (pairs of keys) x (chunks of a row) over the threads
    __shared__ __attribute__((aligned(16))) char k_lds[KEYS * K_ROW];
    __shared__ __attribute__((aligned(16))) char vt_lds[DH * VT_ROW];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int item = blockIdx.x;
    const epara_attn_args a = args[__builtin_amdgcn_readfirstlane(find_attn_group(args, G, item, lane))];
    const int local = item - a.first_item, image = local / a.heads, head = local - image * a.heads;
    const int T = a.tokens, d = a.heads * DH;
    const int n_qb = (T + 15) >> 4;
    const size_t row_bytes = static_cast<size_t>(3 * d) * 2;
    const EPARA_GLOBAL char* qkv = (const EPARA_GLOBAL char*)a.QKV + static_cast<size_t>(image) * T * row_bytes + static_cast<size_t>(head) * DH * 2;

    const int j = lane & 15, g = lane >> 4;
    // wave w takes the query blocks first_qb, first_qb + 8, ...; which waves get a block more rotates with the
    // item, so that two workgroups sharing a compute unit do not put their longer waves on the same SIMDs
    const int first_qb = (wave + item) & (ATTN_WAVES - 1);
    // ---- every load of the workgroup first, so that their latencies overlap: the head's keys and values (a thread
    // takes two neighbouring keys x one 16-byte chunk per step) and this wave's query operands (dims 8 g .. 8 g + 7
    // and 32 + 8 g ..; a query row past the image repeats the last one)
    v4i kv[STAGE_STEPS][2], vv[STAGE_STEPS][2];
#pragma unroll
    for (int it = 0; it < STAGE_STEPS; ++it) {
        const int idx = it * NT_ATTN + tid, chunk = idx & 7;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int key = 2 * (idx >> 3) + e;
            kv[it][e] = v4i{0, 0, 0, 0};
            vv[it][e] = v4i{0, 0, 0, 0};
            if (key < T) {
                const EPARA_GLOBAL char* src = qkv + key * row_bytes + chunk * 16;
                kv[it][e] = *reinterpret_cast<const EPARA_GLOBAL v4i*>(src + static_cast<size_t>(d) * 2);
                vv[it][e] = *reinterpret_cast<const EPARA_GLOBAL v4i*>(src + static_cast<size_t>(d) * 4);
            }
        }
    }
    v4i qf[MAX_QB][2];
#pragma unroll
    for (int i = 0; i < MAX_QB; ++i) {
        const int q = min((first_qb + ATTN_WAVES * i) * 16 + j, T - 1);
        qf[i][0] = *reinterpret_cast<const EPARA_GLOBAL v4i*>(qkv + q * row_bytes + g * 16);
        qf[i][1] = *reinterpret_cast<const EPARA_GLOBAL v4i*>(qkv + q * row_bytes + 64 + g * 16);
    }
    // ---- keys row-major (swizzled), values transposed (two keys = one 32-bit word per head dimension); rows past
    // the image are zeros: their scores are masked, and 0 * 0 is what the second product needs there.  V^T keeps
    // head dimension 16 a + 4 b + r (a, b, r < 4) in row 16 b + 4 a + r: block b of the second product then leaves
    // lane (query, g) with dimensions 16 g + 4 b .. + 3, i.e. 16 consecutive ones over its four blocks.
#pragma unroll
    for (int it = 0; it < STAGE_STEPS; ++it) {
        const int idx = it * NT_ATTN + tid, pair = idx >> 3, chunk = idx & 7;
        if (pair < KEYS / 2) {
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int key = 2 * pair + e;
                *reinterpret_cast<v4i*>(k_lds + key * K_ROW + ((chunk ^ (key & 7)) << 4)) = kv[it][e];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t x0 = static_cast<uint32_t>(vv[it][0][e >> 1]), x1 = static_cast<uint32_t>(vv[it][1][e >> 1]);
                const uint32_t w = e & 1 ? (x0 >> 16) | (x1 & 0xffff0000u) : (x0 & 0xffffu) | (x1 << 16);
                const int row = ((((chunk & 1) << 1) | (e >> 2)) << 4) + ((chunk >> 1) << 2) + (e & 3);     // of dimension 8 chunk + e
                *reinterpret_cast<uint32_t*>(vt_lds + row * VT_ROW + pair * 4) = w;
            }
        }
    }
    __syncthreads();

    const float scale = 1.4426950408889634f * rsqrtf(static_cast<float>(DH));      // scores in units of log 2: exp2 below
    EPARA_GLOBAL char* out = (EPARA_GLOBAL char*)a.O + static_cast<size_t>(image) * T * d * 2 + static_cast<size_t>(head) * DH * 2;
#pragma unroll
    for (int i = 0; i < MAX_QB; ++i) {
        const int qb = first_qb + ATTN_WAVES * i;
        if (qb >= n_qb) break;
        const v4i q0 = qf[i][0], q1 = qf[i][1];
        // ---- S^T, block by block of 16 keys
        v4f s[KB];
#pragma unroll
        for (int b = 0; b < KB; ++b) {
            const int key = b * 16 + j;
            const v4i k0 = *reinterpret_cast<const v4i*>(k_lds + key * K_ROW + ((g ^ (key & 7)) << 4));
            const v4i k1 = *reinterpret_cast<const v4i*>(k_lds + key * K_ROW + (((4 + g) ^ (key & 7)) << 4));
            s[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k0), __builtin_bit_cast(bf16x8, q0), v4f{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
            s[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k1), __builtin_bit_cast(bf16x8, q1), s[b], 0, 0, 0);
        }
        // ---- softmax over the keys of my query: my 4 keys per block, then the lanes j, j + 16, j + 32, j + 48.
        // Keys past the image are masked; the maximum is taken over the raw scores (the scale is positive).
        const int my_keys = T - g * 4;                           // key b * 16 + g * 4 + r exists iff b * 16 + r < my_keys
        float m = -INFINITY;
#pragma unroll
        for (int b = 0; b < KB; ++b) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (b * 16 + r >= my_keys) s[b][r] = -INFINITY;
            m = fmaxf(fmaxf(m, fmaxf(s[b][0], s[b][1])), fmaxf(s[b][2], s[b][3]));
        }
        m = fmaxf(m, __shfl_xor(m, 16));
        m = fmaxf(m, __shfl_xor(m, 32));                         // finite: key 0 exists
        const float ms = m * scale;
        float l = 0.f;
#pragma unroll
        for (int b = 0; b < KB; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                s[b][r] = __builtin_amdgcn_exp2f(fmaf(s[b][r], scale, -ms));          // 2^(scale (s - m)) in (0, 1]; 0 for masked keys
                l += s[b][r];
            }
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        // ---- O^T = V^T P^T, two key blocks per step
        v4f o[DH / 16];
#pragma unroll
        for (int db = 0; db < DH / 16; ++db) o[db] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int p = 0; p < KB / 2; ++p) {
            v4i pb;
            pb[0] = static_cast<int>(pack_bf16(s[2 * p][0], s[2 * p][1]));
            pb[1] = static_cast<int>(pack_bf16(s[2 * p][2], s[2 * p][3]));
            pb[2] = static_cast<int>(pack_bf16(s[2 * p + 1][0], s[2 * p + 1][1]));
            pb[3] = static_cast<int>(pack_bf16(s[2 * p + 1][2], s[2 * p + 1][3]));
#pragma unroll
            for (int db = 0; db < DH / 16; ++db) {
                const char* vrow = vt_lds + (db * 16 + j) * VT_ROW + (p * 32 + g * 4) * 2;
                const v2u lo = *reinterpret_cast<const v2u*>(vrow), hi = *reinterpret_cast<const v2u*>(vrow + 32);
                const v4i va = {static_cast<int>(lo[0]), static_cast<int>(lo[1]), static_cast<int>(hi[0]), static_cast<int>(hi[1])};
                o[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, va), __builtin_bit_cast(bf16x8, pb), o[db], 0, 0, 0);
            }
        }
        // ---- my query's columns 16 g .. 16 g + 15 of this head (block db holds 16 g + 4 db .. + 3): 32 bytes in a row
        if (qb * 16 + j < T) {
            const float inv = 1.f / l;
            EPARA_GLOBAL char* dst = out + static_cast<size_t>(qb * 16 + j) * d * 2 + g * 32;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                v4i pk;
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    pk[2 * k] = static_cast<int>(pack_bf16(o[2 * h + k][0] * inv, o[2 * h + k][1] * inv));
                    pk[2 * k + 1] = static_cast<int>(pack_bf16(o[2 * h + k][2] * inv, o[2 * h + k][3] * inv));
                }
                *reinterpret_cast<EPARA_GLOBAL v4i*>(dst + h * 16) = pk;
            }
        }
    }
}

inline bool misaligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

}  // namespace

extern "C" {

int32_t epara_add_layernorm(const epara_norm_args* h_args, const epara_norm_args* d_args, int32_t G, void* stream)
{
    if (G < 0) return EPARA_ERR_SHAPE;
    if (G == 0) return EPARA_OK;
    if (!h_args || !d_args) return EPARA_ERR_NULL;
    int64_t rows = 0;
    int32_t widest = 8;
    for (int32_t g = 0; g < G; ++g) {
        const epara_norm_args& a = h_args[g];
        if (a.M < 0 || a.d < 8 || a.d > EPARA_NORM_MAX_D || (a.d & 7) || !(a.eps >= 0.f) || !(a.eps < INFINITY)) return EPARA_ERR_SHAPE;
        if (a.first_row != rows) return EPARA_ERR_SHAPE;
        if (a.M > 0 && (!a.X || !a.gamma || !a.beta || !a.Y)) return EPARA_ERR_NULL;
        if (misaligned(a.X, 16) || misaligned(a.R, 16) || misaligned(a.S, 16) || misaligned(a.Y, 16) ||
            misaligned(a.gamma, 16) || misaligned(a.beta, 16)) return EPARA_ERR_ALIGN;
        rows += a.M;
        if (a.M > 0 && a.d > widest) widest = a.d;
        if (rows > INT32_MAX) return EPARA_ERR_SHAPE;
    }
    if (rows == 0) return EPARA_OK;
    const int64_t groups_of_rows = (rows + NT / 64 - 1) / (NT / 64);
    const int grid = static_cast<int>(groups_of_rows < NORM_GRID ? groups_of_rows : NORM_GRID);
    const int per_lane = (widest + 511) >> 9;                    // 16-byte chunks per lane of the widest row
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (per_lane <= 2)      hipLaunchKernelGGL(add_layernorm_kernel<2>, dim3(grid), dim3(NT), 0, s, d_args, G, static_cast<int>(rows));
    else if (per_lane <= 4) hipLaunchKernelGGL(add_layernorm_kernel<4>, dim3(grid), dim3(NT), 0, s, d_args, G, static_cast<int>(rows));
    else if (per_lane <= 8) hipLaunchKernelGGL(add_layernorm_kernel<8>, dim3(grid), dim3(NT), 0, s, d_args, G, static_cast<int>(rows));
    else                    hipLaunchKernelGGL(add_layernorm_kernel<16>, dim3(grid), dim3(NT), 0, s, d_args, G, static_cast<int>(rows));
    return hipGetLastError() == hipSuccess ? EPARA_OK : EPARA_ERR_HIP;
}

int32_t epara_attention(const epara_attn_args* h_args, const epara_attn_args* d_args, int32_t G, void* stream)
{
    if (G < 0) return EPARA_ERR_SHAPE;
    if (G == 0) return EPARA_OK;
    if (!h_args || !d_args) return EPARA_ERR_NULL;
    int64_t items = 0;
    int32_t longest = 1;
    for (int32_t g = 0; g < G; ++g) {
        const epara_attn_args& a = h_args[g];
        if (a.M < 0 || a.tokens < 1 || a.tokens > EPARA_ATTN_MAX_TOKENS || a.heads < 1 || a.head_dim != EPARA_ATTN_HEAD_DIM ||
            a.M % a.tokens != 0 || a.heads > INT32_MAX / (3 * EPARA_ATTN_HEAD_DIM)) return EPARA_ERR_SHAPE;
        if (a.first_item != items) return EPARA_ERR_SHAPE;
        if (a.M > 0 && (!a.QKV || !a.O)) return EPARA_ERR_NULL;
        if (a.M > 0 && a.QKV == a.O) return EPARA_ERR_SHAPE;
        if (misaligned(a.QKV, 16) || misaligned(a.O, 16)) return EPARA_ERR_ALIGN;
        items += static_cast<int64_t>(a.M / a.tokens) * a.heads;
        if (a.M > 0 && a.tokens > longest) longest = a.tokens;
        if (items > INT32_MAX) return EPARA_ERR_SHAPE;
    }
    if (items == 0) return EPARA_OK;
    const int blocks = (longest + 15) / 16;                      // key blocks of the longest image
    const dim3 grid(static_cast<unsigned>(items)), wg(NT_ATTN);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (blocks <= 2)      hipLaunchKernelGGL(attention_kernel<2>, grid, wg, 0, s, d_args, G);
    else if (blocks <= 4) hipLaunchKernelGGL(attention_kernel<4>, grid, wg, 0, s, d_args, G);
    else if (blocks <= 8) hipLaunchKernelGGL(attention_kernel<8>, grid, wg, 0, s, d_args, G);
    else                  hipLaunchKernelGGL(attention_kernel<MAX_KB>, grid, wg, 0, s, d_args, G);
    return hipGetLastError() == hipSuccess ? EPARA_OK : EPARA_ERR_HIP;
}

}  // extern "C"
