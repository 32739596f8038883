// Chains of launches as one kernel: fp8_ffn.
#include "epara_grouped.h"

hipError_t epara_chain_fp8_ffn(const epara_chain_tables& T, const epara_chain_scalars& S, unsigned grid, hipStream_t stream, int64_t* resident)
{
    return chain_kernel_entry<EPARA_FP8_E4M3, true>(T, S, grid, stream, resident);
}
