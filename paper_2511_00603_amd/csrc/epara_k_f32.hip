// fp32 kernels of libepara (grouped launch and chain), the weight packing kernel and a fill kernel.
#include "epara_f32.h"
#include "epara_internal.h"

namespace {

__global__ __launch_bounds__(F32_NT) void grouped_kernel_f32(const epara_group_args* __restrict__ args,
                                                             const epara_tile* __restrict__ tiles,
                                                             const int32_t* __restrict__ order, long n_slots)
{
    f32_body<false>(args, tiles, order, n_slots, nullptr);
}

#define CHAIN_TABLES(i) const epara_group_args* __restrict__ a##i, const epara_tile* __restrict__ t##i, \
                        const int32_t* __restrict__ o##i, const epara_chain_wait* __restrict__ w##i
#define CHAIN_PICK(p, x) ((p) == 0 ? x##0 : (p) == 1 ? x##1 : (p) == 2 ? x##2 : x##3)

__global__ __launch_bounds__(F32_NT) void grouped_chain_kernel_f32(CHAIN_TABLES(0), CHAIN_TABLES(1), CHAIN_TABLES(2), CHAIN_TABLES(3),
                                                                   const epara_chain_scalars S)
{
    chain_ctx c;
    c.waits = nullptr; c.ws = S.ws; c.spin_limit = S.spin_limit; c.counter_base = 0;
    c.pend_group[0] = c.pend_group[1] = -1; c.pend_n[0] = c.pend_n[1] = 0; c.ok_group = -1;
    for (int p = 0; p < S.n_phases; ++p) {
        chain_flush(c);                      // counts of the phase before go to that phase's counters
        c.waits = CHAIN_PICK(p, w);
        c.counter_base = S.counter_base[p];
        c.ok_group = -1;
        f32_body<true>(CHAIN_PICK(p, a), CHAIN_PICK(p, t), CHAIN_PICK(p, o), S.n_slots[p], &c);
    }
    chain_exit(c, S.n_counters);
}

__global__ void fill_words_kernel(uint32_t* p, long n, uint32_t v)
{
    for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += static_cast<long>(gridDim.x) * blockDim.x) p[i] = v;
}

__global__ void copy_word_kernel(const uint32_t* src, uint32_t* dst) { *dst = *src; }

// One 16-byte chunk of the packed weights per thread.
template <int ESZ>
__global__ void pack_kernel(const char* __restrict__ W, int K, int N, char* __restrict__ out, long n_chunks)
{
    constexpr int EPC = 16 / ESZ, KF = 4 * EPC;
    const long idx = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (idx >= n_chunks) return;
    const int KS = ((K + KF - 1) / KF + 3) & ~3;                  // stages per column block, padded to a multiple of four
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

}  // namespace

hipError_t epara_enqueue_f32(unsigned grid, hipStream_t stream, const epara_group_args* args, const epara_tile* tiles,
                             const int32_t* order, long n_slots)
{
    hipLaunchKernelGGL(grouped_kernel_f32, dim3(grid), dim3(F32_NT), 0, stream, args, tiles, order, n_slots);
    return hipGetLastError();
}

hipError_t epara_chain_f32(const epara_chain_tables& T, const epara_chain_scalars& S, unsigned grid, hipStream_t stream, int64_t* resident)
{
    const void* fn = reinterpret_cast<const void*>(&grouped_chain_kernel_f32);
    if (resident) {
        int per_cu = 0, cus = 0, dev = 0;
        if (hipError_t e = hipGetDevice(&dev)) return e;
        if (hipError_t e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) return e;
        if (hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, F32_NT, 0)) return e;
        *resident = static_cast<int64_t>(per_cu) * cus;
        return hipSuccess;
    }
    hipLaunchKernelGGL(grouped_chain_kernel_f32, dim3(grid), dim3(F32_NT), 0, stream,
                       T.args[0], T.tiles[0], T.order[0], T.waits[0], T.args[1], T.tiles[1], T.order[1], T.waits[1],
                       T.args[2], T.tiles[2], T.order[2], T.waits[2], T.args[3], T.tiles[3], T.order[3], T.waits[3], S);
    return hipGetLastError();
}

hipError_t epara_enqueue_fill_words(uint32_t* p, long n, uint32_t v, hipStream_t stream)
{
    hipLaunchKernelGGL(fill_words_kernel, dim3(static_cast<unsigned>(n < 65536 ? (n + 255) / 256 : 256)), dim3(256), 0, stream, p, n, v);
    return hipGetLastError();
}

hipError_t epara_enqueue_copy_word(const uint32_t* src, uint32_t* dst, hipStream_t stream)
{
    hipLaunchKernelGGL(copy_word_kernel, dim3(1), dim3(1), 0, stream, src, dst);
    return hipGetLastError();
}

hipError_t epara_enqueue_pack(int esz, const char* W, int K, int N, char* out, long n_chunks, hipStream_t stream)
{
    const unsigned blocks = static_cast<unsigned>((n_chunks + 255) / 256);
    if (esz == 2) hipLaunchKernelGGL(pack_kernel<2>, dim3(blocks), dim3(256), 0, stream, W, K, N, out, n_chunks);
    else          hipLaunchKernelGGL(pack_kernel<1>, dim3(blocks), dim3(256), 0, stream, W, K, N, out, n_chunks);
    return hipGetLastError();
}
