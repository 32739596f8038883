// Measurement probes of the benchmark (a library of their own, built beside bench.py; not part of
// libepara): what this GPU sustains, so that roofline fractions can be read against measured
// ceilings as well as the data-sheet ones.  Every entry point returns 0 or a hipError_t / -1.
//   probe_read   streams `bytes` (>= 8 KiB, rounded down to 8 KiB per wave step) of d_buf once with
//                n_workgroups workgroups of 256 threads, 16-byte loads, each wave reading consecutive
//                1 KiB chunks: the read bandwidth this GPU sustains.  d_sink: 4 writable bytes.
//   probe_copy   plain copy kernel d_dst[0..bytes) = d_src[0..bytes) (bytes a multiple of 16): a kernel
//                of known HBM traffic against which profiler byte counters are calibrated.
//   probe_mfma   register-resident bf16 MFMA loop: every wave of n_workgroups x 256 threads issues
//                iters x 16 v_mfma_f32_32x32x16_bf16 (16 independent accumulators) on operands taken
//                from d_operands (8 x 256 x 16 bytes).  The sustained rate depends on the operand
//                VALUES (clocks are power limited), so the caller passes data distributed like its
//                workload.  Flops per call = n_workgroups * 4 * iters * 16 * 2*32*32*16.
#include <hip/hip_runtime.h>
#include <stdint.h>


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

int32_t probe_read(const void* d_buf, int64_t bytes, void* d_sink, int32_t n_workgroups, void* stream)
{
    if (!d_buf || !d_sink) return -1;
    if (bytes < 8192 || n_workgroups <= 0) return -1;
    if (reinterpret_cast<uintptr_t>(d_buf) & 15u) return -1;
    (void)hipGetLastError();
    hipLaunchKernelGGL(read_kernel, dim3(static_cast<unsigned>(n_workgroups)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const v4i*>(d_buf), static_cast<long>(bytes / 1024), static_cast<int*>(d_sink));
    return static_cast<int32_t>(hipGetLastError());
}

int32_t probe_copy(const void* d_src, void* d_dst, int64_t bytes, void* stream)
{
    if (!d_src || !d_dst) return -1;
    if (bytes < 16) return -1;
    if ((reinterpret_cast<uintptr_t>(d_src) | reinterpret_cast<uintptr_t>(d_dst)) & 15u) return -1;
    (void)hipGetLastError();
    hipLaunchKernelGGL(copy_kernel, dim3(4096), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const v4i*>(d_src), static_cast<v4i*>(d_dst), static_cast<long>(bytes / 16));
    return static_cast<int32_t>(hipGetLastError());
}

int32_t probe_mfma(const void* d_operands, int32_t iters, void* d_sink, int32_t n_workgroups, void* stream)
{
    if (!d_operands || !d_sink) return -1;
    if (iters <= 0 || n_workgroups <= 0) return -1;
    if (reinterpret_cast<uintptr_t>(d_operands) & 15u) return -1;
    (void)hipGetLastError();
    hipLaunchKernelGGL(mfma_kernel, dim3(static_cast<unsigned>(n_workgroups)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const v4i*>(d_operands), iters, static_cast<float*>(d_sink));
    return static_cast<int32_t>(hipGetLastError());
}

}  // extern "C"
