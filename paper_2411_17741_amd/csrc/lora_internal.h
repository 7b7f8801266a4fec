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

// Token ids of N rows of a tile in one round of lookups (none for a tile of consecutive tokens).  Rows past the
// tile's last count as its last, the rows of an empty tile as token `dead`.  (A conditional lookup per row is a
// branch per row in a kernel, and after each the compiler waits for every load and store still outstanding.)
template <int N>
inline __host__ __device__ void tile_tokens_of(const int32_t *tok_list, const DevItem &it, const int (&ti)[N], int32_t dead,
                                               int (&tok)[N])
{
    if (it.n_tok <= 0) {
#pragma unroll
        for (int i = 0; i < N; ++i) tok[i] = dead;
    } else if (it.consecutive) {
#pragma unroll
        for (int i = 0; i < N; ++i) tok[i] = it.tok0 + (ti[i] < it.n_tok ? ti[i] : it.n_tok - 1);
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) tok[i] = tok_list[it.tok_off + (ti[i] < it.n_tok ? ti[i] : it.n_tok - 1)];
    }
}

// GEMV work item: a batch of up to GEMV_BATCH tokens of one slot, named directly so that the kernels
// reach their data with one lookup.  A shrink item stands for GEMV_SHRINK_ROWS stored rank rows from
// `a` on (stored rows past the rank hold zeros, so an item is always whole); an expand item for one
// run of gemv_expand_width(rank) columns in every super-chunk of the projection, `a` being the
// run's offset inside the super-chunk in units of 64 columns.  Items name no projection: a launch
// runs them for every projection of its group.  Kernels and lora_plan_dump read `a` through the
// routines below.
constexpr int GEMV_BATCH = 4;              // tokens one GEMV work item handles
constexpr int GEMV_SHRINK_ROWS = 4;        // rank rows of a shrink item
constexpr int GEMV_SUPER_COLS = 1024;      // an expand item stands for one run of columns in every super-chunk of this width
struct GemvItem {
    int32_t tok[GEMV_BATCH];  // token ids, -1 = unused; used ones come first
    int32_t row;              // first storage row of the slot
    int32_t rank;
    int32_t a;
    float alpha;              // the cache entry's own factor
};
static_assert(sizeof(GemvItem) == 32, "items are read with one 32-byte scalar load");

// columns one expand wavefront covers: 64 times the largest power of two that keeps it within 16 KB of Bp
inline __host__ __device__ int32_t gemv_expand_width(int32_t rank)
{
    const int32_t q = 128 / rank_storage(rank);
    return q >= 16 ? 1024 : q >= 8 ? 512 : q >= 4 ? 256 : q >= 2 ? 128 : 64;
}
inline __host__ __device__ int32_t gemv_pack_shrink(int32_t j0) { return j0; }
inline __host__ __device__ int32_t gemv_pack_expand(int32_t col_in_super) { return col_in_super / 64; }
// stored rank rows [j0, j0 + n) of a shrink item
inline __host__ __device__ void gemv_shrink_rows(const GemvItem &it, int32_t &j0, int32_t &n)
{
    j0 = it.a;
    n = GEMV_SHRINK_ROWS;
}
// output columns [c0, c1) of expand item `it` in super-chunk `sc` of a projection h_out wide (empty if c0 >= c1)
inline __host__ __device__ void gemv_expand_cols(const GemvItem &it, int32_t sc, int32_t h_out, int32_t &c0, int32_t &c1)
{
    c0 = sc * GEMV_SUPER_COLS + it.a * 64;
    const int32_t end = c0 + gemv_expand_width(it.rank), super_end = (sc + 1) * GEMV_SUPER_COLS;
    c1 = end < super_end ? end : super_end;
    if (c1 > h_out) c1 = h_out;
}

// One GEMV launch serves up to GEMV_MAX_PROJS projections that read the same activations (q, k, v;
// gate, up): block and unit numbers map to (projection, item) by the two routines below, which the
// kernels and lora_plan_dump share.
constexpr int GEMV_MAX_PROJS = 4;
struct GemvProj {
    const char *proj_base;    // device: first slab of this (layer, projection)
    int64_t row_bytes;        // (h_in + h_out) * element size
    void *y;                  // device [T][h_out], in/out
    float *y32;               // when set, the update s.v.B goes there as fp32 ([token][h_out]) instead of into y
    unsigned long long *vw;   // hand-over words of this projection's intermediate (see gemv_kernels.hip)
    int32_t h_out;
    int32_t pad;
};
// What a wavefront needs to find its work item, apart from the rest: the kernels take it as leading
// scalar arguments, which the hardware hands over in registers at wavefront start (no load to wait for
// before the item's own load can go out).
struct GemvMap {
    const GemvItem *gs, *ge;  // device: shrink and expand items
    uint32_t n_gs;
    uint32_t n_proj_phase;    // n_proj | phase << 8; phase 0: shrink blocks then expand blocks in one launch; 1: shrink only; 2: expand only
    int32_t unit_end[GEMV_MAX_PROJS];      // expand units of projections 0 .. p (entries past the group repeat the last)
    uint32_t n_super_packed;               // super-chunks of projection p, ceil(h_out / GEMV_SUPER_COLS) (< 256), in byte p
    uint32_t super_magic[GEMV_MAX_PROJS];  // ceil(2^32 / n_super) (unused when n_super == 1)
};
struct GemvArgs {
    const void *x;            // device [T][h_in]
    int32_t *fault;           // raised when a bounded wait gives up
    int32_t h_in, n_ge;
    uint32_t epoch;           // one launch: the number its hand-over words carry (never 0); 0: two launches, no waiting
    float scale;
    GemvProj p[GEMV_MAX_PROJS];
};
// floor(v / n) for v < 2^24 and n <= 255 with magic = ceil(2^32 / n), n > 1
inline __host__ __device__ uint32_t gemv_div(uint32_t v, uint32_t n, uint32_t magic)
{
    return n == 1 ? v : (uint32_t)(((uint64_t)v * magic) >> 32);
}
inline uint32_t gemv_magic(uint32_t n) { return n > 1 ? (uint32_t)((((uint64_t)1 << 32) + n - 1) / n) : 0; }
// one of four values by an index 0..3 (as selects: an array indexed by a run-time number would live in scratch memory on the device)
template <typename T> inline __host__ __device__ T gemv_sel4(uint32_t i, T v0, T v1, T v2, T v3)
{
    return i == 0 ? v0 : (i == 1 ? v1 : (i == 2 ? v2 : v3));
}
// Shrink block b of a launch with n_proj * n_gs shrink blocks -> (item, projection).  Block b runs on
// XCD b % 8, each XCD behind its own L2: XCD j takes a run of consecutive (item, projection) pairs,
// items in list order with their projections side by side, the i-th pair of the run as block 8i + j --
// the items of a token batch and all their projections read the batch's x rows, which are then
// fetched from memory by one XCD instead of eight.
inline __host__ __device__ void gemv_shrink_block(uint32_t b, uint32_t n_gs, uint32_t n_proj, uint32_t &item, uint32_t &proj)
{
    const uint32_t nb = n_gs * n_proj, j = b & 7;
    const uint32_t pos = j * (nb >> 3) + (j < (nb & 7) ? j : (nb & 7)) + (b >> 3);
    item = n_proj == 1 ? pos : (n_proj == 2 ? pos >> 1 : (n_proj == 4 ? pos >> 2 : gemv_div(pos, 3u, 0x55555556u)));
    proj = pos - item * n_proj;
}
// Expand unit u (over all projections of the launch) -> (projection, item, super-chunk)
inline __host__ __device__ void gemv_expand_unit(uint32_t u, const GemvMap &m, uint32_t &proj, uint32_t &item, uint32_t &sc)
{
    proj = (u >= (uint32_t)m.unit_end[0]) + (u >= (uint32_t)m.unit_end[1]) + (u >= (uint32_t)m.unit_end[2]);  // < n_proj for u < unit_end[n_proj - 1]
    const uint32_t r = u - gemv_sel4<uint32_t>(proj, 0u, (uint32_t)m.unit_end[0], (uint32_t)m.unit_end[1], (uint32_t)m.unit_end[2]);
    const uint32_t n_super = (m.n_super_packed >> (8 * proj)) & 0xffu;
    item = gemv_div(r, n_super, gemv_sel4(proj, m.super_magic[0], m.super_magic[1], m.super_magic[2], m.super_magic[3]));
    sc = r - item * n_super;
}

// Arguments common to the apply kernels of one (layer, projection).
struct ApplyArgs {
    const char *proj_base;    // device: first slab of this (layer, projection)
    int64_t row_bytes;        // (h_in + h_out) * element size
    const int32_t *tok_list;  // device
    const void *x;            // device [T][h_in]
    void *y;                  // device [T][h_out], in/out
    float *v;                 // device, rows of v_stride floats, one per token: the tile path's shrink result, kept as
                              // bf16 entries s.v[j] (scale and alpha applied) at the front of the token's row
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
// GEMV shrink and expand of the group's projections: phase 0 as one launch (a.epoch != 0: the expand
// wavefronts wait for the hand-over words to carry that number), phases 1 and 2 as two
hipError_t launch_gemv(int dtype, const GemvMap &m, const GemvArgs &a, hipStream_t st, const KernelTimer *tm);
// bytes of one projection's hand-over words for max_tokens tokens
size_t gemv_handover_bytes(int dtype, int64_t max_tokens);
// zeroes the hand-over words of tokens toks[0 .. n) (device list) in `vw`
hipError_t launch_gemv_clear(int dtype, unsigned long long *vw, const int32_t *toks, int n, hipStream_t st);
// Tile shrink.  Its work is the sequence of all tiles' k ranges, every tile's range divided into `quanta`
// equal parts (a part is a whole number of the kernel's k stages for every projection of the cache).  A plan
// cuts that sequence into n_runs runs of about equal cost (a tile's cost per part: its x rows plus its At
// rows); run r is worked on by one block per projection of the launch, all blocks of a launch being
// resident at once (two per compute unit), so that the launch ends when a run ends.  A run covers a tail of
// its first tile, whole tiles, and a head of its last tile; a piece that is not a whole tile leaves a partial
// sum in the scratch rows of (run, first or last piece) and mfma_reduce_kernel adds a tile's pieces up.
// Cuts lie on part boundaries at least SHRINK_MIN_PARTS parts from a tile's ends and from each other, or on a
// tile boundary; the last runs of a table may be empty (the table is padded to a multiple of 8 runs).
struct ShrinkCut {  // where run r starts (it ends where run r + 1 starts; entry n_runs = {n_tiles, 0})
    int32_t tile;
    int32_t part;   // 0 <= part < quanta
};
struct ShrinkSum {  // per tile, for the reduce: its pieces' partial sums
    int32_t first_slot;  // scratch slot of the first piece; piece j > 0 lies in slot 2 * (first_slot / 2 + j)
    int32_t n_pieces;    // 1: the tile was worked on whole, the shrink wrote the result itself
};
constexpr int SHRINK_MIN_PARTS = 2;
constexpr int SHRINK_SLOT_ROWS = LORA_TILE_TOKENS;  // rows (of v_stride floats) of one partial-sum slot
// scratch slot of the piece of tile `tile` in run `run` that starts in tile `first_tile`
inline __host__ __device__ int32_t shrink_slot(int32_t run, int32_t first_tile, int32_t tile) { return 2 * run + (tile != first_tile); }
// k stages (of stage_k elements) before part boundary `part` of a row of h_in elements
inline __host__ __device__ int32_t shrink_part_stage(int32_t part, int32_t quanta, int32_t h_in, int32_t stage_k)
{
    const int32_t n_st = (h_in + stage_k - 1) / stage_k;
    return (int32_t)(((int64_t)part * n_st + quanta / 2) / quanta);
}
constexpr int SHRINK_STAGE_K = 128;
// The projections one tile-shrink launch serves (they read the same x): slab base and row pitch,
// destination of the intermediate, scratch for the partial sums (2 * n_runs slots of SHRINK_SLOT_ROWS rows).
constexpr int MAX_SHRINK_PROJS = 4;
struct ShrinkProjs {
    int n;
    int n_runs, quanta;       // n_runs: a multiple of 8 (run r is worked on by XCD r / (n_runs / 8))
    int any_pieces;           // some tile is worked on in pieces: the reduce launch is needed
    const ShrinkCut *cuts;    // device, n_runs + 1
    const ShrinkSum *sums;    // device, n_tiles
    const char *proj_base[MAX_SHRINK_PROJS];
    int64_t row_bytes[MAX_SHRINK_PROJS];
    float *v[MAX_SHRINK_PROJS];     // as ApplyArgs::v
    float *part[MAX_SHRINK_PROJS];  // fp32 partial sums of the tiles worked on in pieces
};
// proj_base, row_bytes and v of `a` are ignored (taken from ps)
hipError_t launch_mfma_shrink(const ApplyArgs &a, const ShrinkProjs &ps, const DevItem *tiles, int n_tiles, hipStream_t st,
                              const KernelTimer *tm);
hipError_t launch_mfma_expand(const ApplyArgs &a, const DevItem *tiles, int n_tiles, hipStream_t st, const KernelTimer *tm);
// y = x . Wt^T + adapter update for row tiles (tiles of the plan, then plain runs of the other tokens:
// rank 0); a.tok_list must be the list the row tiles index; a.v holds the shrink results
hipError_t launch_zero_rows(void *y, const int32_t *toks, int n, int h_out, hipStream_t st);  // y bf16 [..][h_out]
// The tiles of the grid's last, partly filled round are split along k over several blocks when
// split_scratch (device, linear_split_bytes() bytes for this shape) and split_flags (device, zero between
// launches, one per split-off part) have room; fault: raised when the bounded wait for a part gives up.
size_t linear_split_bytes(int n_rt, int h_in, int h_out, int n_cu);
hipError_t launch_linear_tiles(const ApplyArgs &a, const void *Wt, const DevItem *row_tiles, int n_rt, void *split_scratch,
                               size_t split_scratch_bytes, uint32_t *split_flags, int n_split_flags, int32_t *fault, int n_cu,
                               hipStream_t st, const KernelTimer *tm);
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
