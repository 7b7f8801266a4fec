// Internal declarations shared by the host side and the gfx950 kernels of liblora_cache.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lora_cache.h"

namespace lora {

// Arguments common to the four apply kernels of one (layer, projection).
struct ApplyArgs {
    const char *layer_base;   // device: first slab of this layer
    const int64_t *slot_off;  // device: [n_slots] byte offset of the slot's slab of this projection
    const int32_t *tok_list;  // device
    const void *x;            // device [T][h_in]
    void *y;                  // device [T][h_out], in/out
    float *v;                 // device [max_tokens][v_stride] shrink result
    int32_t h_in, h_out, v_stride;
    float scale;
};

// Pool layout of one slab (adapter of rank r, rs = r rounded up to a multiple of 8):
//   At [rs][h_in]          rank-major: row j holds column j of A, contiguous along h_in
//   Bp [rs/8][h_out][8]    rank-packed: the 8 ranks of a granule are contiguous per output column
// Rows r..rs-1 are zero.  Only rs*(h_in+h_out) elements are ever read, whatever the slot's class.
inline __host__ __device__ int32_t rank_storage(int32_t r) { return (r + 7) & ~7; }

// launches (all asynchronous on `st`); dtype is LORA_F32 or LORA_BF16
hipError_t launch_gemv_shrink(int dtype, const ApplyArgs &a, const lora_item_t *items, int n_items, hipStream_t st);
hipError_t launch_gemv_expand(int dtype, const ApplyArgs &a, const lora_item_t *items, int n_items, hipStream_t st);
hipError_t launch_mfma_shrink(const ApplyArgs &a, const lora_item_t *tiles, int n_tiles, int k_splits, hipStream_t st);
hipError_t launch_mfma_expand(const ApplyArgs &a, const lora_item_t *tiles, int n_tiles, hipStream_t st);
hipError_t launch_zero_f32(float *p, size_t n, hipStream_t st);
// staged [h_in][r] / [r][h_out] -> slab layout
hipError_t launch_repack(int dtype, const void *stage_A, const void *stage_B, void *slab, int32_t h_in, int32_t h_out,
                         int32_t rank, hipStream_t st);

}  // namespace lora
