// Measurement helpers of libepara (not part of the forward path): what this GPU sustains, so
// that roofline fractions can be read against measured ceilings as well as the data-sheet ones.
//   epara_probe_read   streams a buffer once (every wave reads consecutive 1 KiB chunks)
//   epara_probe_copy   plain copy kernel of known size (calibrates the HBM traffic counters)
//   epara_probe_mfma   register-resident 32x32x16 bf16 MFMA loop on caller-provided operand data
//                      (the sustained matrix rate depends on the operand values: power-limited)
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "epara.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__global__ __launch_bounds__(256) void read_kernel(const v4i* __restrict__ p, long n_chunks, int* sink)
{
    const long wave = static_cast<long>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    const long n_waves = static_cast<long>(gridDim.x) * 4;
    const int lane = threadIdx.x & 63;
    v4i acc = {0, 0, 0, 0};
    for (long c = wave * 8; c + 8 <= n_chunks; c += n_waves * 8) {
        v4i v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = p[(c + u) * 64 + lane];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x5a5a1234) sink[0] = 1;     // keeps the loads alive
}

__global__ __launch_bounds__(256) void copy_kernel(const v4i* __restrict__ src, v4i* __restrict__ dst, long n)
{
    for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += static_cast<long>(gridDim.x) * blockDim.x)
        dst[i] = src[i];
}

// 16 accumulators of 32x32, operands rotate so that the data keeps changing like a real K loop.
__global__ __launch_bounds__(256) void mfma_kernel(const v4i* __restrict__ ops, int iters, float* sink)
{
    v4i a[4], b[4];
    for (int i = 0; i < 4; ++i) { a[i] = ops[i * 256 + threadIdx.x]; b[i] = ops[(4 + i) * 256 + threadIdx.x]; }
    v16f c[4][4];
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 4; ++j) for (int v = 0; v < 16; ++v) c[i][j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                c[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[j]), c[i][j], 0, 0, 0);
        const v4i t = a[0]; a[0] = a[1]; a[1] = a[2]; a[2] = a[3]; a[3] = t;
    }
    float s = 0.f;
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 4; ++j) s += c[i][j][0];
    if (s == 1234.5f) sink[0] = s;
}

}  // namespace

extern "C" {

int32_t epara_probe_read(const void* d_buf, int64_t bytes, void* d_sink, int32_t n_workgroups, void* stream)
{
    if (!d_buf || !d_sink) return EPARA_ERR_NULL;
    if (bytes < 8192 || n_workgroups <= 0) return EPARA_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(d_buf) & 15u) return EPARA_ERR_ALIGN;
    (void)hipGetLastError();
    hipLaunchKernelGGL(read_kernel, dim3(static_cast<unsigned>(n_workgroups)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const v4i*>(d_buf), static_cast<long>(bytes / 1024), static_cast<int*>(d_sink));
    return hipGetLastError() == hipSuccess ? EPARA_OK : EPARA_ERR_HIP;
}

int32_t epara_probe_copy(const void* d_src, void* d_dst, int64_t bytes, void* stream)
{
    if (!d_src || !d_dst) return EPARA_ERR_NULL;
    if (bytes < 16) return EPARA_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(d_src) | reinterpret_cast<uintptr_t>(d_dst)) & 15u) return EPARA_ERR_ALIGN;
    (void)hipGetLastError();
    hipLaunchKernelGGL(copy_kernel, dim3(4096), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const v4i*>(d_src), static_cast<v4i*>(d_dst), static_cast<long>(bytes / 16));
    return hipGetLastError() == hipSuccess ? EPARA_OK : EPARA_ERR_HIP;
}

int32_t epara_probe_mfma(const void* d_operands, int32_t iters, void* d_sink, int32_t n_workgroups, void* stream)
{
    if (!d_operands || !d_sink) return EPARA_ERR_NULL;
    if (iters <= 0 || n_workgroups <= 0) return EPARA_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(d_operands) & 15u) return EPARA_ERR_ALIGN;
    (void)hipGetLastError();
    hipLaunchKernelGGL(mfma_kernel, dim3(static_cast<unsigned>(n_workgroups)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const v4i*>(d_operands), iters, static_cast<float*>(d_sink));
    return hipGetLastError() == hipSuccess ? EPARA_OK : EPARA_ERR_HIP;
}

}  // extern "C"
