// Grouped launches of libepara: fp8_gated kernels (mixed and panel-only).
#include "epara_grouped.h"

hipError_t epara_enqueue_fp8_gated(int panel_only, unsigned grid, hipStream_t stream, const epara_group_args* args, const epara_tile* tiles,
                            const int32_t* order, long n_slots, int out_dtype, int narrow, uint32_t* split_ws, int n_split, int n_panel_split, int first_panel_split)
{
    return enqueue_grouped<EPARA_FP8_E4M3, true>(panel_only, grid, stream, args, tiles, order, n_slots, out_dtype, narrow, split_ws, n_split, n_panel_split, first_panel_split);
}
