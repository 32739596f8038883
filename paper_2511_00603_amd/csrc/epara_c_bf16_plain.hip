// Chains of launches as one kernel: bf16_plain.
#include "epara_grouped.h"

hipError_t epara_chain_bf16_plain(const epara_chain_tables& T, const epara_chain_scalars& S, unsigned grid, hipStream_t stream, int64_t* resident)
{
    return chain_kernel_entry<EPARA_BF16, false>(T, S, grid, stream, resident);
}
