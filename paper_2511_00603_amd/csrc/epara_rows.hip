// libepara: batch forming around the grouped forward (Sec. 3.1 BS / MF of the paper: the rows of
// many requests become one ragged batch per service and the result rows go back to them).
//
//   epara_copy_segments            gather / scatter of row runs (a batched copy)
//   epara_quantize_segments_e4m3   gather + dynamic per-tensor E4M3 quantisation
//   epara_patch_scales             device-side scale products into the group arguments
//
// All of it is bound by HBM traffic: every source byte is read once (twice when quantising:
// once for the maximum, once for the codes) and every destination byte written once.  A
// workgroup of 256 threads moves 16-KiB chunks with 16-byte accesses per lane (a wave
// instruction covers 1 KiB of consecutive memory); chunk c belongs to the last segment whose
// first_chunk is <= c, found by bisection (the value is the same for all lanes: scalar loads).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "epara.h"
#include "epara_cast.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
#define EPARA_GLOBAL __attribute__((address_space(1)))

constexpr int NT = 256;
constexpr int64_t CHUNK = 16384;
constexpr int MAX_GRID = 256 * 16;       // workgroups: enough waves to keep every HBM channel busy

__device__ __forceinline__ int64_t find_segment(const epara_segment* __restrict__ segs, int64_t n, int64_t c)
{
    int64_t lo = 0, hi = n - 1;            // invariant: first_chunk[lo] <= c
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (segs[mid].first_chunk <= c) lo = mid; else hi = mid - 1;
    }
    return lo;
}

__global__ __launch_bounds__(NT) void copy_segments_kernel(const epara_segment* __restrict__ segs, int64_t n, int64_t n_chunks)
{
    for (int64_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
        const epara_segment sg = segs[find_segment(segs, n, c)];
        const int64_t base = (c - sg.first_chunk) * CHUNK;
        const EPARA_GLOBAL char* src = (const EPARA_GLOBAL char*)sg.src + base;
        EPARA_GLOBAL char* dst = (EPARA_GLOBAL char*)sg.dst + base;
        const int64_t left = sg.bytes - base;
        v4i v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t off = (i * NT + threadIdx.x) * 16;
            if (off < left) v[i] = *reinterpret_cast<const EPARA_GLOBAL v4i*>(src + off);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t off = (i * NT + threadIdx.x) * 16;
            if (off < left) *reinterpret_cast<EPARA_GLOBAL v4i*>(dst + off) = v[i];
        }
    }
}

// |x| as an unsigned integer that orders like the magnitude (fp32 bit pattern without its sign;
// a bf16 is the upper half of one).
template <int SRC>
__device__ __forceinline__ uint32_t max_abs_bits(const v4i& v)
{
    uint32_t m = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t u = static_cast<uint32_t>(v[j]);
        if constexpr (SRC == EPARA_F32) {
            m = max(m, u & 0x7fffffffu);
        } else {
            m = max(m, (u << 16) & 0x7fffffffu);
            m = max(m, u & 0x7fff0000u);
        }
    }
    return m;
}

template <int SRC>
__global__ __launch_bounds__(NT) void amax_segments_kernel(const epara_segment* __restrict__ segs, int64_t n, int64_t n_chunks,
                                                           unsigned int* __restrict__ amax_bits)
{
    // A workgroup keeps the maximum of its chunks in registers while they belong to one service and
    // publishes it when the service changes or its work ends: atomics on one address serialise,
    // one per chunk would cost more than reading the data.
    __shared__ uint32_t part[NT / 64];
    uint32_t m = 0;
    int group = -1;
    auto publish = [&]() {
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) m = max(m, static_cast<uint32_t>(__shfl_xor(static_cast<int>(m), d)));
        if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
        __syncthreads();
        if (threadIdx.x == 0) {
            const uint32_t w = max(max(part[0], part[1]), max(part[2], part[3]));
            // integer maximum: the order of arrival cannot matter; skipped when it cannot raise the value
            if (w > __hip_atomic_load(amax_bits + group, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(amax_bits + group, w);
        }
        __syncthreads();
        m = 0;
    };
    for (int64_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
        const epara_segment sg = segs[find_segment(segs, n, c)];
        if (sg.group != group) {
            if (group >= 0) publish();
            group = sg.group;
        }
        const int64_t base = (c - sg.first_chunk) * CHUNK;
        const EPARA_GLOBAL char* src = (const EPARA_GLOBAL char*)sg.src + base;
        const int64_t left = sg.bytes - base;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t off = (i * NT + threadIdx.x) * 16;
            if (off < left) {
                const v4i v = *reinterpret_cast<const EPARA_GLOBAL v4i*>(src + off);
                m = max(m, max_abs_bits<SRC>(v));
            }
        }
    }
    if (group >= 0) publish();
}

__global__ void clear_kernel(unsigned int* p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

__device__ __forceinline__ float scale_of(float amax) { return amax > 0.f ? amax / 448.f : 1.f; }

template <int SRC>
__global__ __launch_bounds__(NT) void quantize_segments_kernel(const epara_segment* __restrict__ segs, int64_t n, int64_t n_chunks,
                                                               const float* __restrict__ amax, float* __restrict__ scale, int G)
{
    constexpr int ESZ = SRC == EPARA_F32 ? 4 : 2;
    if (blockIdx.x == 0)
        for (int g = threadIdx.x; g < G; g += NT) scale[g] = scale_of(amax[g]);
    for (int64_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
        const epara_segment sg = segs[find_segment(segs, n, c)];
        const float inv = 1.f / scale_of(amax[sg.group]);      // codes = RNE(x * (1 / scale)), as the forward path's epilogue does
        const int64_t base = (c - sg.first_chunk) * CHUNK;
        const EPARA_GLOBAL char* src = (const EPARA_GLOBAL char*)sg.src + base;
        EPARA_GLOBAL char* dst = (EPARA_GLOBAL char*)sg.dst + base / ESZ;
        const int64_t left = sg.bytes - base;
        v4i v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t off = (i * NT + threadIdx.x) * 16;
            if (off < left) v[i] = *reinterpret_cast<const EPARA_GLOBAL v4i*>(src + off);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t off = (i * NT + threadIdx.x) * 16;
            if (off >= left) continue;
            if constexpr (SRC == EPARA_F32) {
                *reinterpret_cast<EPARA_GLOBAL uint32_t*>(dst + off / 4) =
                    epara_cast::f32x4_to_e4m3(__int_as_float(v[i][0]) * inv, __int_as_float(v[i][1]) * inv, __int_as_float(v[i][2]) * inv, __int_as_float(v[i][3]) * inv);
            } else {
                float f[8];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t u = static_cast<uint32_t>(v[i][j]);
                    f[2 * j] = __uint_as_float(u << 16) * inv;
                    f[2 * j + 1] = __uint_as_float(u & 0xffff0000u) * inv;
                }
                v2u pk;
                pk[0] = epara_cast::f32x4_to_e4m3(f[0], f[1], f[2], f[3]);
                pk[1] = epara_cast::f32x4_to_e4m3(f[4], f[5], f[6], f[7]);
                *reinterpret_cast<EPARA_GLOBAL v2u*>(dst + off / 2) = pk;
            }
        }
    }
}

__global__ void patch_scales_kernel(epara_group_args* __restrict__ args, int G, const float* __restrict__ sx,
                                    const float* __restrict__ sw, const float* __restrict__ sw2, const float* __restrict__ sout)
{
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= G) return;
    args[g].scale = sx[g] * sw[g];
    if (sw2) args[g].scale2 = sx[g] * sw2[g];
    if (sout) args[g].out_inv_scale = 1.f / sout[g];
}

int32_t check_segments(const epara_segment* h, const epara_segment* d, int64_t n, int64_t n_chunks, int32_t G)
{
    if (n < 0 || n_chunks < 0) return EPARA_ERR_SHAPE;
    if (n == 0) return n_chunks == 0 ? EPARA_OK : EPARA_ERR_SHAPE;
    if (!h || !d) return EPARA_ERR_NULL;
    int64_t chunks = 0;
    for (int64_t i = 0; i < n; ++i) {
        const epara_segment& s = h[i];
        if (s.bytes < 0 || s.first_chunk != chunks) return EPARA_ERR_SHAPE;
        if (G >= 0 && (s.group < 0 || s.group >= G)) return EPARA_ERR_SHAPE;
        if (s.bytes > 0 && (!s.src || !s.dst)) return EPARA_ERR_NULL;
        if ((s.bytes & 15) || (reinterpret_cast<uintptr_t>(s.src) & 15) || (reinterpret_cast<uintptr_t>(s.dst) & 15))
            return EPARA_ERR_ALIGN;
        chunks += (s.bytes + CHUNK - 1) / CHUNK;
    }
    return chunks == n_chunks ? EPARA_OK : EPARA_ERR_SHAPE;
}

inline int grid_for(int64_t n_chunks) { return static_cast<int>(n_chunks < MAX_GRID ? n_chunks : MAX_GRID); }

}  // namespace

extern "C" {

int32_t epara_copy_segments(const epara_segment* h_segments, const epara_segment* d_segments,
                            int64_t n_segments, int64_t n_chunks, void* stream)
{
    if (int32_t st = check_segments(h_segments, d_segments, n_segments, n_chunks, -1)) return st;
    if (n_chunks == 0) return EPARA_OK;
    hipLaunchKernelGGL(copy_segments_kernel, dim3(grid_for(n_chunks)), dim3(NT), 0, static_cast<hipStream_t>(stream),
                       d_segments, n_segments, n_chunks);
    return hipGetLastError() == hipSuccess ? EPARA_OK : EPARA_ERR_HIP;
}

int32_t epara_quantize_segments_e4m3(const epara_segment* h_segments, const epara_segment* d_segments,
                                     int64_t n_segments, int64_t n_chunks, int32_t G, int32_t src_dtype,
                                     float* d_amax, float* d_scale, void* stream)
{
    if (G < 0) return EPARA_ERR_SHAPE;
    if (src_dtype != EPARA_F32 && src_dtype != EPARA_BF16) return EPARA_ERR_DTYPE;
    if (int32_t st = check_segments(h_segments, d_segments, n_segments, n_chunks, G)) return st;
    if (G == 0) return EPARA_OK;
    if (!d_amax || !d_scale) return EPARA_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 small((G + 255) / 256), grid(static_cast<int>(n_chunks < 1024 ? (n_chunks > 0 ? n_chunks : 1) : 1024));
    // the maxima are cleared by a kernel, not a memset: a caller may capture this stream in a graph
    hipLaunchKernelGGL(clear_kernel, small, dim3(256), 0, s, reinterpret_cast<unsigned int*>(d_amax), G);
    if (n_chunks > 0) {
        if (src_dtype == EPARA_F32)
            hipLaunchKernelGGL(amax_segments_kernel<EPARA_F32>, grid, dim3(NT), 0, s, d_segments, n_segments, n_chunks,
                               reinterpret_cast<unsigned int*>(d_amax));
        else
            hipLaunchKernelGGL(amax_segments_kernel<EPARA_BF16>, grid, dim3(NT), 0, s, d_segments, n_segments, n_chunks,
                               reinterpret_cast<unsigned int*>(d_amax));
    }
    // the quantising kernel also writes the scales (workgroup 0); with no data it runs for that alone
    const dim3 qgrid(n_chunks > 0 ? grid_for(n_chunks) : 1);
    if (src_dtype == EPARA_F32)
        hipLaunchKernelGGL(quantize_segments_kernel<EPARA_F32>, qgrid, dim3(NT), 0, s, d_segments, n_segments, n_chunks, d_amax, d_scale, G);
    else
        hipLaunchKernelGGL(quantize_segments_kernel<EPARA_BF16>, qgrid, dim3(NT), 0, s, d_segments, n_segments, n_chunks, d_amax, d_scale, G);
    return hipGetLastError() == hipSuccess ? EPARA_OK : EPARA_ERR_HIP;
}

int32_t epara_patch_scales(epara_group_args* d_args, int32_t G, const float* d_sx, const float* d_sw,
                           const float* d_sw2, const float* d_sout, void* stream)
{
    if (G < 0) return EPARA_ERR_SHAPE;
    if (G == 0) return EPARA_OK;
    if (!d_args || !d_sx || !d_sw) return EPARA_ERR_NULL;
    hipLaunchKernelGGL(patch_scales_kernel, dim3((G + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                       d_args, G, d_sx, d_sw, d_sw2, d_sout);
    return hipGetLastError() == hipSuccess ? EPARA_OK : EPARA_ERR_HIP;
}

}  // extern "C"
