// Host-side seams between the translation units of libepara (one per kernel family, so that they
// compile side by side).  Nothing here is part of the C ABI.
#ifndef EPARA_INTERNAL_H
#define EPARA_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "epara.h"

#define EPARA_HIDDEN __attribute__((visibility("hidden")))

struct epara_chain_scalars {
    long n_slots[EPARA_MAX_CHAIN_PHASES];
    int out_dtype[EPARA_MAX_CHAIN_PHASES], narrow[EPARA_MAX_CHAIN_PHASES], counter_base[EPARA_MAX_CHAIN_PHASES];
    uint32_t* ws;
    uint32_t spin_limit;
    int n_phases, n_counters;
};

struct epara_chain_tables {
    const epara_group_args* args[EPARA_MAX_CHAIN_PHASES];
    const epara_tile* tiles[EPARA_MAX_CHAIN_PHASES];
    const int32_t* order[EPARA_MAX_CHAIN_PHASES];
    const epara_chain_wait* waits[EPARA_MAX_CHAIN_PHASES];
};

// One grouped launch; dtype = EPARA_BF16 / EPARA_FP8_E4M3; panel_only: the tile table holds no streaming tile.
EPARA_HIDDEN hipError_t epara_enqueue_bf16_plain(int panel_only, unsigned grid, hipStream_t, const epara_group_args*, const epara_tile*, const int32_t*, long n_slots, int out_dtype, int narrow, uint32_t* split_ws, int n_split, int n_panel_split, int first_panel_split);
EPARA_HIDDEN hipError_t epara_enqueue_bf16_gated(int panel_only, unsigned grid, hipStream_t, const epara_group_args*, const epara_tile*, const int32_t*, long n_slots, int out_dtype, int narrow, uint32_t* split_ws, int n_split, int n_panel_split, int first_panel_split);
EPARA_HIDDEN hipError_t epara_enqueue_fp8_plain(int panel_only, unsigned grid, hipStream_t, const epara_group_args*, const epara_tile*, const int32_t*, long n_slots, int out_dtype, int narrow, uint32_t* split_ws, int n_split, int n_panel_split, int first_panel_split);
EPARA_HIDDEN hipError_t epara_enqueue_fp8_gated(int panel_only, unsigned grid, hipStream_t, const epara_group_args*, const epara_tile*, const int32_t*, long n_slots, int out_dtype, int narrow, uint32_t* split_ws, int n_split, int n_panel_split, int first_panel_split);
EPARA_HIDDEN hipError_t epara_enqueue_f32(unsigned grid, hipStream_t, const epara_group_args*, const epara_tile*, const int32_t*, long n_slots);

// Chain kernels.  resident != NULL: no launch, *resident = workgroups of that kernel the current device holds at once.
EPARA_HIDDEN hipError_t epara_chain_bf16_plain(const epara_chain_tables&, const epara_chain_scalars&, unsigned grid, hipStream_t, int64_t* resident);
EPARA_HIDDEN hipError_t epara_chain_bf16_ffn(const epara_chain_tables&, const epara_chain_scalars&, unsigned grid, hipStream_t, int64_t* resident);
EPARA_HIDDEN hipError_t epara_chain_fp8_plain(const epara_chain_tables&, const epara_chain_scalars&, unsigned grid, hipStream_t, int64_t* resident);
EPARA_HIDDEN hipError_t epara_chain_fp8_ffn(const epara_chain_tables&, const epara_chain_scalars&, unsigned grid, hipStream_t, int64_t* resident);
EPARA_HIDDEN hipError_t epara_chain_f32(const epara_chain_tables&, const epara_chain_scalars&, unsigned grid, hipStream_t, int64_t* resident);

EPARA_HIDDEN hipError_t epara_enqueue_fill_words(uint32_t* p, long n, uint32_t v, hipStream_t);
EPARA_HIDDEN hipError_t epara_enqueue_copy_word(const uint32_t* src, uint32_t* dst, hipStream_t);
EPARA_HIDDEN hipError_t epara_enqueue_pack(int esz, const char* W, int K, int N, char* out, long n_chunks, hipStream_t);

#endif
