// Chains of launches as one kernel: bf16_ffn.
#include "epara_grouped.h"

hipError_t epara_chain_bf16_ffn(const epara_chain_tables& T, const epara_chain_scalars& S, unsigned grid, hipStream_t stream, int64_t* resident)
{
    return chain_kernel_entry<EPARA_BF16, true>(T, S, grid, stream, resident);
}
