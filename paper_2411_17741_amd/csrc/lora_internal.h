// Internal declarations shared by the host side and the gfx950 kernels of liblora_cache.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "lora_cache.h"

namespace lora {

// Pool layout.  Every slot owns `rs_class` consecutive *storage rows* (rs = rank rounded up
// to a multiple of 8); a slot's first row is the same number in every projection, so a slab
// is found without a table:
//     slab(layer, proj, slot) = pool + layer*layer_stride + proj_off[proj] + row(slot) * row_bytes(proj)
//     row_bytes(proj) = (h_in + h_out) * element size
// Inside a slab of an adapter of rank r (rs = rank_storage(r)):
//   At [rs][h_in]          rank-major: row j holds column j of A, contiguous along h_in
//   Bp [rs/8][h_out][8]    rank-packed: the 8 ranks of a granule are contiguous per output column
// Rows r..rs-1 are zero.  Only rs*(h_in+h_out) elements are ever read, whatever the slot's class.
inline __host__ __device__ int32_t rank_storage(int32_t r) { return (r + 7) & ~7; }

// Work item as the kernels read it (the public lora_item_t with the slot resolved).
struct DevItem {
    int32_t tok_off, n_tok;  // tokens: tok_list[tok_off .. tok_off+n_tok)
    int32_t row;             // first storage row of the slot
    int32_t rank;
    int32_t a;               // as in lora_item_t
    int32_t consecutive;     // 1: the tokens are tok0, tok0+1, ... (a prompt's tile): no lookup in tok_list at all
    float alpha;             // the cache entry's own factor
    int32_t tok0;            // tok_list[tok_off], so one-token items need no second lookup
};
static_assert(sizeof(DevItem) == sizeof(lora_item_t), "device items are uploaded in place of lora_item_t");
// token id of row ti (0 <= ti < n_tok) of a tile (tile kernels and lora_plan_dump alike)
inline __host__ __device__ int32_t tile_token_of(const int32_t *tok_list, const DevItem &it, int32_t ti)
{
    return (it.consecutive || ti == 0) ? it.tok0 + ti : tok_list[it.tok_off + ti];
}

// GEMV work item: a batch of up to GEMV_BATCH tokens of one slot, named directly so that
// the kernels reach their data with one lookup.  `a` packs, for a shrink item, the first rank
// row (bits 0-7) and the number of rows (bits 8+); for an expand item the column offset in the
// super-chunk divided by 64.  Kernels and lora_plan_dump read `a` through the two routines below.
constexpr int GEMV_BATCH = 4;              // tokens one GEMV work item handles
constexpr int GEMV_SHRINK_ROWS = 4;        // rank rows of a shrink item
constexpr int GEMV_SUPER_COLS = 1024;      // an expand item stands for one run of columns in every super-chunk of this width
struct GemvItem {
    int32_t tok[GEMV_BATCH];  // token ids, -1 = unused
    int32_t row;              // first storage row of the slot
    int32_t rank;
    int32_t a;
    float alpha;              // expand: the cache entry's own factor
};
static_assert(sizeof(GemvItem) == 32, "items are read with two 16-byte loads");

// columns one expand wavefront covers: 16 KB of Bp whatever the rank
inline __host__ __device__ int32_t gemv_expand_width(int32_t rank)
{
    const int32_t q = 128 / rank_storage(rank);
    return 64 * (q > 1 ? q : 1);
}
inline __host__ __device__ int32_t gemv_pack_shrink(int32_t j0, int32_t n_rows) { return j0 | (n_rows << 8); }
inline __host__ __device__ int32_t gemv_pack_expand(int32_t col_in_super) { return col_in_super / 64; }
// rank rows [j0, j0 + n) of a shrink item
inline __host__ __device__ void gemv_shrink_rows(const GemvItem &it, int32_t &j0, int32_t &n)
{
    j0 = it.a & 0xff;
    n = it.a >> 8;
}
// output columns [c0, c1) of expand item `it` in super-chunk `sc` of a projection h_out wide (empty if c0 >= c1)
inline __host__ __device__ void gemv_expand_cols(const GemvItem &it, int32_t sc, int32_t h_out, int32_t &c0, int32_t &c1)
{
    c0 = sc * GEMV_SUPER_COLS + (it.a & 0xf) * 64;
    const int32_t end = c0 + gemv_expand_width(it.rank), super_end = (sc + 1) * GEMV_SUPER_COLS;
    c1 = end < super_end ? end : super_end;
    if (c1 > h_out) c1 = h_out;
}

// Arguments common to the apply kernels of one (layer, projection).
struct ApplyArgs {
    const char *proj_base;    // device: first slab of this (layer, projection)
    int64_t row_bytes;        // (h_in + h_out) * element size
    const int32_t *tok_list;  // device
    const void *x;            // device [T][h_in]
    void *y;                  // device [T][h_out], in/out
    float *v;                 // device [max_tokens][v_stride] shrink result
    int32_t h_in, h_out, v_stride;
    float scale;
    // when set, the GEMV expand writes its term s.v.B there as fp32 ([token][h_out]) instead of adding it to y,
    // and linear_tiles_kernel takes the term of its GEMV rows from there
    float *y32 = nullptr;
};

// Optional per-kernel timing: when a launch gets a KernelTimer it asks it for an event pair and
// launches through hipExtLaunchKernelGGL, which stamps the pair with the kernel's own start and
// end (no bracketing commands in the stream, so kernels are neither serialised nor padded).
struct KernelTimer {
    void *ctx;
    void (*pair)(void *ctx, int kind, hipEvent_t *start, hipEvent_t *stop);
};

template <typename K, typename... A>
inline void launch_k(const KernelTimer *tm, int kind, K kernel, dim3 grid, dim3 block, hipStream_t st, A... args)
{
    hipEvent_t s = nullptr, e = nullptr;
    if (tm) tm->pair(tm->ctx, kind, &s, &e);
    if (s && e) hipExtLaunchKernelGGL(kernel, grid, block, 0, st, s, e, 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, 0, st, args...);
}

// launches (all asynchronous on `st`); dtype is LORA_F32 or LORA_BF16; tm may be null
hipError_t launch_gemv_shrink(int dtype, const ApplyArgs &a, const GemvItem *items, int n_items, hipStream_t st,
                              const KernelTimer *tm);
hipError_t launch_gemv_expand(int dtype, const ApplyArgs &a, const GemvItem *items, int n_items, hipStream_t st,
                              const KernelTimer *tm);
// shrink and expand in one launch: expand wavefronts load their slab part at once and then poll
// the intermediate, which travels as 64-bit words {epoch, fp32 bits} in vtag (device, max_tokens
// rows of v_stride words, never holding a number >= epoch on entry); epoch != 0; `fault` (device
// int32) is set if a wait gives up
hipError_t launch_gemv_fused(int dtype, const ApplyArgs &a, const GemvItem *gs, int n_gs, const GemvItem *ge, int n_ge,
                             unsigned long long *vtag, uint32_t epoch, int32_t *fault, hipStream_t st, const KernelTimer *tm);
// The projections one tile-shrink launch serves (they read the same x): slab base and row pitch,
// destination of the intermediate, scratch for k-split partials (splits * n_tile_tok rows of
// v_stride floats each, unused when the launch does not split).
constexpr int MAX_SHRINK_PROJS = 4;
struct ShrinkProjs {
    int n;
    // tiles [xcd_tile[j], xcd_tile[j+1]) are worked on by the blocks of XCD j: contiguous runs (tiles
    // of a prompt share At, which then stays in that XCD's L2) of about equal cost (a tile of rank
    // 128 takes twice as long as one of rank 16; with equal counts the XCD that got a long
    // high-rank prompt finished last by a factor of two)
    int xcd_tile[9];
    const char *proj_base[MAX_SHRINK_PROJS];
    int64_t row_bytes[MAX_SHRINK_PROJS];
    float *v[MAX_SHRINK_PROJS];
    float *part[MAX_SHRINK_PROJS];
};
// n_tile_tok = tokens of all tiles (the leading part of tok_list); proj_base, row_bytes and v of
// `a` are ignored (taken from ps)
hipError_t launch_mfma_shrink(const ApplyArgs &a, const ShrinkProjs &ps, const DevItem *tiles, int n_tiles, int n_tile_tok,
                              int k_splits, hipStream_t st, const KernelTimer *tm);
int mfma_shrink_splits(int h_in, int want);  // k ranges the shrink launch will really use
hipError_t launch_mfma_expand(const ApplyArgs &a, const DevItem *tiles, int n_tiles, hipStream_t st, const KernelTimer *tm);
// y = x . Wt^T + adapter update for row tiles (tiles of the plan, then plain runs of the other tokens:
// rank 0); a.tok_list must be the list the row tiles index; a.v holds the shrink results
hipError_t launch_zero_rows(void *y, const int32_t *toks, int n, int h_out, hipStream_t st);  // y bf16 [..][h_out]
hipError_t launch_linear_tiles(const ApplyArgs &a, const void *Wt, const DevItem *row_tiles, int n_rt, hipStream_t st,
                               const KernelTimer *tm);
// A [h_in][r] / B [r][h_out] (16-byte aligned; device memory, or pinned host memory as the device
// sees it: from_host) -> slab layout
hipError_t launch_repack(int dtype, const void *src_A, const void *src_B, void *slab, int32_t h_in, int32_t h_out,
                         int32_t rank, bool from_host, hipStream_t st);
// the same for up to REPACK_MAX_PARTS parts of one adapter in one launch (unit_end, r, rs are set by the launcher)
constexpr int REPACK_MAX_PARTS = 32;
struct RepackPart {
    const void *A, *B;
    void *slab;
    int32_t h_in, h_out, unit_end, pad;
};
struct RepackTable {
    RepackPart p[REPACK_MAX_PARTS];
    int32_t n, r, rs, pad;
};
hipError_t launch_repack_parts(int dtype, RepackTable &t, int32_t rank, bool from_host, hipStream_t st);

}  // namespace lora
