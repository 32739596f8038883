// Chains of launches as one kernel: fp8_plain.
#include "epara_grouped.h"

hipError_t epara_chain_fp8_plain(const epara_chain_tables& T, const epara_chain_scalars& S, unsigned grid, hipStream_t stream, int64_t* resident)
{
    return chain_kernel_entry<EPARA_FP8_E4M3, false>(T, S, grid, stream, resident);
}
