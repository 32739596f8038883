// fp32 groups of libepara: plain FMA tiles.
#ifndef EPARA_F32_H
#define EPARA_F32_H

#include "epara_device.h"

namespace {

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

}  // namespace

#endif
