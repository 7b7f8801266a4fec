// Matrix-core path of the batched LoRA apply for gfx950 (bf16 in, fp32 accumulate): tiles of
// up to 64 tokens that share one cache slot -- prompt segments, or the pooled decode tokens
// of a hot adapter.  Built on v_mfma_f32_16x16x32_bf16; operand layout of that instruction:
//   A (16 x 32): lane l holds row l%16,  k = 8*(l/16) .. +7
//   B (32 x 16): lane l holds col l%16,  k = 8*(l/16) .. +7
//   D (16 x 16): lane l holds col l%16,  rows 4*(l/16) .. +3
// Because a contraction does not care about the order of k, both kernels give every lane
// group a k range that makes the lane's global loads contiguous and use the same range for
// both operands.
//
//   shrink:  V[tile][rank] = X[tile][k-range] . At^T        (split over k ranges of h_in)
//   expand:  Y[tile][cols]^T += Bp[cols][rank] . (s.V)^T     (split over column ranges)
//
// (paper section 3.1: the two adapter products and the aggregation into the base output.)
#include <algorithm>
#include <type_traits>

#include "lora_device.h"

namespace lora {

namespace {
constexpr int VS_ROW = LORA_MAX_RANK * 2 + 16;  // bytes per token row of the staged V tile (padded)
}  // namespace

// ---------------------------------------------------------------------------------------
// shrink.  Block = 4 wavefronts on one tile and one k range, walked in stages of 128 k.
//  - x, the HBM stream, goes through an LDS ring of three stages: every thread fetches four
//    16-byte pieces per stage with a wavefront instruction covering 4 token rows x 256
//    contiguous bytes, two stages ahead of the one being multiplied (so two stages of loads are
//    in flight in registers while a third waits ready in LDS), one barrier per stage.  Rows are
//    padded by 16 bytes, which puts the 16 rows of an A-operand read in distinct banks.
//  - At, which comes out of L2 and is shared by all tiles of a segment, is loaded into registers one
//    stage ahead -- the four lanes of a quad on one rank row (64-byte requests; in the operand's own
//    order, with neighbouring lanes in different rows, the same bytes cost the load path 1.7 times
//    as long) -- and put in operand order by a lane permutation before the products.
//  - From 4 rank blocks (of 16) up, wavefront w owns rank blocks w and w+4 for the whole k range
//    and writes its part of V itself.  Below that, the wavefronts split the four MFMA k steps of
//    a stage instead, each covering all rank blocks, and their partials are summed through LDS.
//  - The launch's work -- every tile's k range -- is cut into runs of about equal cost, one block per run
//    (and projection), all blocks resident at once: a block walks the pieces of its run, a piece being a k
//    range of one tile.  A piece that is not a whole tile leaves a partial sum in the scratch slot of its run
//    and mfma_reduce_kernel adds a tile's pieces up.  (With one block per tile and a fixed number of k ranges
//    the launch ended when the XCD with the most or the costliest tiles did: a timeline of the prefill
//    configuration showed half of the blocks done at 15 us and the last at 26 us.)
// Blocks are numbered so that consecutive runs (same tiles, same segment, same At) fall on one XCD (blocks
// b, b + 8, ... run on XCD b % 8).
// One launch can serve several projections that read the same x (q, k, v; gate, up).
// ---------------------------------------------------------------------------------------
namespace {
constexpr int SK = SHRINK_STAGE_K;      // k elements per stage
constexpr int XROW = SK * 2 + 16;       // bytes per token row of a stage in LDS
constexpr int NSTAGE = 3;
}  // namespace

// Every global load below is unconditional, from an address clamped into the tensor, and what
// must not count is zeroed where x is written to LDS (zero x rows and zero x tail columns make
// whatever At held there irrelevant).  Loads under a condition would be compiled into branches,
// and the wait counters cannot be tracked across those: every stage would then wait for all
// outstanding loads and the prefetch distance would collapse to nothing.
// token id of row ti (>= 0) of a tile
__device__ __forceinline__ int tile_token(const ApplyArgs &a, const DevItem &it, int ti)
{
    return tile_token_of(a.tok_list, it, ti);
}

// token ids of N rows of a tile at once (rows past the tile's last count as its last)
template <int N>
__device__ __forceinline__ void tile_tokens(const ApplyArgs &a, const DevItem &it, const int (&ti)[N], int (&tok)[N])
{
    tile_tokens_of(a.tok_list, it, ti, it.tok0, tok);
}

template <bool NSPLIT, int NBW>  // NBW: rank blocks (of 16) a wavefront works on
__device__ __forceinline__ void mfma_shrink_body(const ApplyArgs &a, const DevItem &it, int k_begin, int k_end, int phase,
                                                 float *part, unsigned char (*xs)[LORA_TILE_TOKENS * XROW])
{
    constexpr int NKW = NSPLIT ? 4 : 1;  // MFMA k steps of a stage a wavefront works on
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int rs = rank_storage(it.rank);
    const int n_st = (k_end - k_begin + SK - 1) / SK;
    const int k_last = a.h_in - 8;  // last 16-byte piece of a row

    const __bf16 *At = reinterpret_cast<const __bf16 *>(a.proj_base + (int64_t)it.row * a.row_bytes);
    const __bf16 *x = static_cast<const __bf16 *>(a.x);

    // k offset of stage st.  The walk over k starts at a different stage in every block, so that
    // blocks running side by side do not all pull the same column window (rows lie h_in apart)
    auto stage_k = [&](int st) {
        // (the prefetches run up to three stages past the end: they re-read the last stage, which is
        // still in L1/L2 -- wrapped round to the first stages they came from memory again, +43 % of x
        // for a block of seven stages)
        int s = min(st, n_st - 1) + phase;
        s -= s >= n_st ? n_st : 0;
        return k_begin + s * SK;
    };

    // loader: rows 16w + 4i + lane/16, piece lane%16 (8 elements)
    const int lp = lane & 15;
    const __bf16 *xg[4];
    int lds_off[4];
    bool x_ok[4];
    {
        int row[4], tok[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) row[i] = 16 * w + 4 * i + (lane >> 4);
        tile_tokens(a, it, row, tok);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x_ok[i] = row[i] < it.n_tok;
            xg[i] = x + (size_t)tok[i] * a.h_in;
            lds_off[i] = row[i] * XROW + lp * 16;
        }
    }
    // At operands: block slot q -> rank block nbq; rows past the stored rank are clamped (their
    // results are never written)
    // A B operand wants, in lane (m, g), rank row m and k chunk g of the step: 16 rows x 64 bytes per load
    // instruction with neighbouring lanes in different rows, the costliest shape for the load path.  The same
    // 16 x 64 bytes are therefore fetched with the four lanes of a quad on one row (lane l: row l/4, chunk
    // l%4 -- a 64-byte request per quad) and put in operand order by a lane permutation on the way to the
    // products (ds_bpermute: lane (m, g) takes the registers of lane 4m + g).
    int nbq[NBW];
    const __bf16 *ag[NBW];
#pragma unroll
    for (int q = 0; q < NBW; ++q) {
        nbq[q] = NSPLIT ? w + 4 * q : q;
        ag[q] = At + (size_t)min(16 * nbq[q] + (lane >> 2), rs - 1) * a.h_in;
    }
    const int perm_src = 4 * (4 * m + g);  // byte address of the source lane, as ds_bpermute takes it
    const int ks0 = NSPLIT ? 0 : w;  // first MFMA k step of a stage for this wavefront

    uint4 xr[2][4];
    auto load_x = [&](int st, uint4(&d)[4]) {
        const int k = min(stage_k(st) + lp * 8, k_last);
#pragma unroll
        for (int i = 0; i < 4; ++i) d[i] = *reinterpret_cast<const uint4 *>(xg[i] + k);
    };
    auto store_x = [&](int slot, int st, const uint4(&d)[4]) {
        const bool k_ok = stage_k(st) + lp * 8 < k_end;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<uint4 *>(&xs[slot][lds_off[i]]) = (x_ok[i] && k_ok) ? d[i] : make_uint4(0, 0, 0, 0);
    };
    uint4 br[2][NBW][NKW];
    auto load_at = [&](int st, uint4(&d)[NBW][NKW]) {
        const int k = stage_k(st) + 8 * (lane & 3);
#pragma unroll
        for (int q = 0; q < NBW; ++q)
#pragma unroll
            for (int j = 0; j < NKW; ++j) d[q][j] = *reinterpret_cast<const uint4 *>(ag[q] + min(k + 32 * (ks0 + j), k_last));
    };
    auto operand_of = [&](const uint4 &r) {
        uint4 o;
        o.x = __builtin_amdgcn_ds_bpermute(perm_src, r.x);
        o.y = __builtin_amdgcn_ds_bpermute(perm_src, r.y);
        o.z = __builtin_amdgcn_ds_bpermute(perm_src, r.z);
        o.w = __builtin_amdgcn_ds_bpermute(perm_src, r.w);
        return __builtin_bit_cast(bf16x8, o);
    };

    floatx4 acc[4][NBW];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int q = 0; q < NBW; ++q) acc[mb][q] = floatx4{0.f, 0.f, 0.f, 0.f};

    load_x(0, xr[0]);
    load_x(1, xr[1]);
    load_at(0, br[0]);
    store_x(0, 0, xr[0]);
    load_x(2, xr[0]);
    __syncthreads();

    // one stage; CUR = st % 2 and SLOT = st % 3 are compile-time constants so that the staging
    // arrays stay in registers and the ring slots are fixed addresses
    auto stage = [&](auto cur_tag, auto slot_tag, int st) {
        constexpr int CUR = decltype(cur_tag)::value;
        constexpr int SLOT = decltype(slot_tag)::value;
        load_at(st + 1, br[CUR ^ 1]);  // At of the next stage, then this stage's products
        const unsigned char *xb = xs[SLOT];
        bf16x8 bop[NBW][NKW];
#pragma unroll
        for (int q = 0; q < NBW; ++q)
#pragma unroll
            for (int j = 0; j < NKW; ++j) bop[q][j] = operand_of(br[CUR][q][j]);
#pragma unroll
        for (int j = 0; j < NKW; ++j) {
            const int ks = ks0 + j;
#pragma unroll
            for (int mb = 0; mb < 4; ++mb) {
                const bf16x8 av = *reinterpret_cast<const bf16x8 *>(&xb[(16 * mb + m) * XROW + (4 * ks + g) * 16]);
#pragma unroll
                for (int q = 0; q < NBW; ++q) acc[mb][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bop[q][j], acc[mb][q], 0, 0, 0);
            }
        }
        // stage st+1 goes to LDS (its buffer was last read two barriers ago), stage st+3 is requested
        store_x((SLOT + 1) % NSTAGE, st + 1, xr[CUR ^ 1]);
        load_x(st + 3, xr[CUR ^ 1]);
        __syncthreads();
    };
    // (the walk leaves through a break after its last stage: with every stage under a condition of its own a
    // stage can be reached past a skipped one as far as the compiler can tell, the load counts it merges at
    // such a join are the smallest of both ways, and every wait for x then also waited for the requests of
    // the stage before -- the two-stage lead of x was one)
    for (int st = 0;; st += 6) {
        stage(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, st);
        if (st + 1 >= n_st) break;
        stage(std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{}, st + 1);
        if (st + 2 >= n_st) break;
        stage(std::integral_constant<int, 0>{}, std::integral_constant<int, 2>{}, st + 2);
        if (st + 3 >= n_st) break;
        stage(std::integral_constant<int, 1>{}, std::integral_constant<int, 0>{}, st + 3);
        if (st + 4 >= n_st) break;
        stage(std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{}, st + 4);
        if (st + 5 >= n_st) break;
        stage(std::integral_constant<int, 1>{}, std::integral_constant<int, 2>{}, st + 5);
        if (st + 6 >= n_st) break;
    }

    // Where the rows go.  The tile's whole k range: the result itself, into the rows of v that belong to the
    // tile's tokens; else this piece's partial sum, one row per row of the tile (mfma_reduce_kernel adds the
    // pieces up).  The row numbers are all fetched before the first store: a lookup between two stores makes
    // the second wait for the first to be acknowledged (loads and stores share the counter, which can only
    // be waited down), 0.3 us each -- 10 us for the 32 stores of a rank-128 piece
    float *const out = part ? part : a.v;
    auto rows_of = [&](int mb, int (&rows)[4]) {
#pragma unroll
        for (int r = 0; r < 4; ++r) rows[r] = 16 * mb + 4 * g + r;
        if (part) return;
        const int ti[4] = {rows[0], rows[1], rows[2], rows[3]};
        tile_tokens(a, it, ti, rows);
    };
    // (a whole tile's result goes out as the expand takes it: scaled and rounded to bf16, rows of the same pitch)
    const float s_v = a.scale * it.alpha;
    __bf16 *const out16 = reinterpret_cast<__bf16 *>(a.v);
    auto write_v = [&](int mb, const int (&rows)[4], int q, const floatx4 &val) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int ti = 16 * mb + 4 * g + r, jr = 16 * nbq[q] + m;
            if (ti < it.n_tok && jr < it.rank) {
                if (part) out[(size_t)rows[r] * a.v_stride + jr] = val[r];
                else out16[(size_t)rows[r] * (2 * a.v_stride) + jr] = (__bf16)(s_v * val[r]);
            }
        }
    };
    if (NSPLIT) {
        int rows[4][4];
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) rows_of(mb, rows[mb]);
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int q = 0; q < NBW; ++q) write_v(mb, rows[mb], q, acc[mb][q]);
    } else {
        // the four wavefronts hold partial sums over k: park them in the (now idle) x ring and let
        // wavefront w add up and write token block w
        float *red = reinterpret_cast<float *>(&xs[0][0]);  // [wave][mb][q][r][lane], at most 4*4*3*4*64*4 B = 48 KB
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int q = 0; q < NBW; ++q)
#pragma unroll
                for (int r = 0; r < 4; ++r) red[(((w * 4 + mb) * NBW + q) * 4 + r) * 64 + lane] = acc[mb][q][r];
        int rows[4];
        rows_of(w, rows);
        __syncthreads();
#pragma unroll
        for (int q = 0; q < NBW; ++q) {
            floatx4 sum = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int src = 0; src < 4; ++src)
#pragma unroll
                for (int r = 0; r < 4; ++r) sum[r] += red[(((src * 4 + w) * NBW + q) * 4 + r) * 64 + lane];
            write_v(w, rows, q, sum);
        }
    }
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void mfma_shrink_kernel(const ShrinkCut *__restrict__ cuts, const DevItem *__restrict__ tiles,
                                                          int runs_per_xcd, int n_proj, int quanta, int n_tiles, ApplyArgs a,
                                                          ShrinkProjs ps)
{
    __shared__ __attribute__((aligned(16))) unsigned char xs[NSTAGE][LORA_TILE_TOKENS * XROW];
    static_assert(sizeof(xs) >= 4 * 4 * 3 * 4 * 64 * 4, "the sum over the wavefronts' k parts reuses the x ring");

    // XCD j = blockIdx % 8 works on the runs [j * runs_per_xcd, (j + 1) * runs_per_xcd); its i-th block on
    // (run, projection) number i, projection innermost: the blocks that read the same part of x for the
    // projections of a group are neighbours in the dispatch order of one XCD and walk k in the same order, so
    // that x is fetched from memory once and found in L2 by the others
    const int xcd = (int)blockIdx.x & 7, local = (int)blockIdx.x >> 3;
    const int run = xcd * runs_per_xcd + local / n_proj, pj = local % n_proj;
    const ShrinkCut from = cuts[run], to = cuts[run + 1];
    a.proj_base = ps.proj_base[pj];
    a.row_bytes = ps.row_bytes[pj];
    a.v = ps.v[pj];
    const int last_tile = min(to.part > 0 ? to.tile : to.tile - 1, n_tiles - 1);
    for (int tile = from.tile; tile <= last_tile; ++tile) {
        const int lo = tile == from.tile ? from.part : 0, hi = tile == to.tile ? to.part : quanta;
        if (lo >= hi) continue;  // (an empty run)
        const DevItem it = tiles[tile];
        const int k_begin = shrink_part_stage(lo, quanta, a.h_in, SK) * SK;
        const int k_end = min(a.h_in, shrink_part_stage(hi, quanta, a.h_in, SK) * SK);
        const int n_st = (k_end - k_begin + SK - 1) / SK;
        const int phase = (int)(((unsigned)(run + tile) * 5u) % (unsigned)n_st);
        float *my_part = (lo == 0 && hi == quanta)
                             ? nullptr
                             : ps.part[pj] + (size_t)shrink_slot(run, from.tile, tile) * SHRINK_SLOT_ROWS * a.v_stride;
        const int NB = (it.rank + 15) >> 4;
        if (NB > 4) mfma_shrink_body<true, 2>(a, it, k_begin, k_end, phase, my_part, xs);
        else if (NB == 4) mfma_shrink_body<true, 1>(a, it, k_begin, k_end, phase, my_part, xs);
        else if (NB == 3) mfma_shrink_body<false, 3>(a, it, k_begin, k_end, phase, my_part, xs);
        else if (NB == 2) mfma_shrink_body<false, 2>(a, it, k_begin, k_end, phase, my_part, xs);
        else mfma_shrink_body<false, 1>(a, it, k_begin, k_end, phase, my_part, xs);
        __syncthreads();  // the next piece reuses the ring
    }
}

// V[token][0..rank) = sum over the tile's pieces of their partial sums, for the tiles worked on in pieces.
// (Atomic adds into V instead cost about 30 us per launch: device-scope fp32 atomics execute at the memory side.)
__global__ __launch_bounds__(256) void mfma_reduce_kernel(ApplyArgs a, ShrinkProjs ps, const DevItem *__restrict__ tiles)
{
    // 8 blocks per tile (and projection of the group: blockIdx.y), 8 tokens each; a thread sums one
    // float4 column of one token
    const int tile = blockIdx.x >> 3;
    const ShrinkSum sm = ps.sums[tile];
    const DevItem it = tiles[tile];  // (requested together with sm: one trip to memory, not two)
    const int ti = (blockIdx.x & 7) * 8 + (threadIdx.x >> 5), j4 = threadIdx.x & 31;
    if ((sm.n_pieces < 2) | (ti >= it.n_tok) | (j4 * 4 >= rank_storage(it.rank))) return;  // entries past the rank are never used
    const size_t slot_f4 = (size_t)SHRINK_SLOT_ROWS * (a.v_stride >> 2);
    const float4 *src = reinterpret_cast<const float4 *>(ps.part[blockIdx.y]) + (size_t)ti * (a.v_stride >> 2) + j4;
    // four pieces at a time: their loads are issued together (one after the other, a tile in seven pieces took
    // seven trips to memory: 6.5 us per launch on the stress configuration), and only the loads that are needed (loads of a
    // padded batch cost the mixed configuration, two to three pieces per tile, 1 to 2 us)
    float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
    auto piece = [&](int pc) __attribute__((always_inline)) {
        return src[(size_t)(pc == 0 ? sm.first_slot : 2 * ((sm.first_slot >> 1) + pc)) * slot_f4];
    };
    auto add = [&](const float4 &v) __attribute__((always_inline)) { sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w; };
    for (int p0 = 0; p0 < sm.n_pieces; p0 += 4) {
        const int n = sm.n_pieces - p0;  // the same for the whole block: the branches below are scalar
        if (n >= 4) {
            const float4 v0 = piece(p0), v1 = piece(p0 + 1), v2 = piece(p0 + 2), v3 = piece(p0 + 3);
            add(v0); add(v1); add(v2); add(v3);
        } else if (n == 3) {
            const float4 v0 = piece(p0), v1 = piece(p0 + 1), v2 = piece(p0 + 2);
            add(v0); add(v1); add(v2);
        } else if (n == 2) {
            const float4 v0 = piece(p0), v1 = piece(p0 + 1);
            add(v0); add(v1);
        } else {
            add(piece(p0));
        }
    }
    // the sum goes out as the expand takes it: scaled and rounded to bf16 (rows of the same pitch as the fp32 ones)
    const float s_v = a.scale * it.alpha;
    typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
    bf16x4_t o;
    o[0] = (__bf16)(s_v * sum.x), o[1] = (__bf16)(s_v * sum.y), o[2] = (__bf16)(s_v * sum.z), o[3] = (__bf16)(s_v * sum.w);
    reinterpret_cast<bf16x4_t *>(reinterpret_cast<__bf16 *>(ps.v[blockIdx.y]) + (size_t)tile_token(a, it, ti) * (2 * a.v_stride))[j4] = o;
}

// ---------------------------------------------------------------------------------------
// expand.  Block = 4 wavefronts, tile of up to 64 tokens x (128 * n_pass) columns in passes of
// 128 columns (the launcher picks n_pass: long column runs per block amortise the staging of V
// when there are many tiles, short ones keep the chip full when there are few); wavefront w owns token half w&1 and column half w>>1 of a pass (32 tokens x 64
// columns).  The scaled V tile is staged once in LDS as bf16.  The product is formed
// transposed (rows = output columns, columns = tokens): MFMA row r of column block b is column
// 16b + r, so the 16 lanes of a Bp operand load read 256 contiguous bytes.
// The read-modify-write of base_out does not use the MFMA register layout (a lane would touch
// 16 bytes of each of many rows, and every 128-byte line would be fetched by two instructions,
// which stalls L1 on the second): the wavefront parks its fp32 products in LDS and goes over
// base_out with 8 lanes per token row, whole 128-byte lines per instruction, for the load (issued
// one pass ahead), the add and the store.
// Register use is held to three blocks per CU (the V operands are re-read from LDS in every pass
// rather than kept): with two, short launches of a few hundred blocks leave CUs idle at the end.
// ---------------------------------------------------------------------------------------
namespace {
constexpr int CS_ROW = 64 * 4 + 16;  // bytes per token row of a wavefront's parked products (padded)
}

// KS: MFMA k steps of 32 ranks.  As in the shrink, global loads are unconditional from clamped
// addresses: rank chunks past the stored rank re-read the last stored chunk and meet zeros in V.
template <int KS>
__device__ __forceinline__ void mfma_expand_body(const ApplyArgs &a, const DevItem &it, int col_run, int n_pass, unsigned char *vs,
                                                 unsigned char (*cs)[32 * CS_ROW])
{
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int th = w & 1, ch = w >> 1;
    const int rs = rank_storage(it.rank), rs8 = rs >> 3;
    const __bf16 *Bp = reinterpret_cast<const __bf16 *>(a.proj_base + (int64_t)it.row * a.row_bytes) + (size_t)rs * a.h_in;
    __bf16 *y = static_cast<__bf16 *>(a.y);

    // read-modify-write layout: instruction i covers token rows 32*th + 8*i + lane/8, 8 columns at 8*(lane%8)
    const int rt = lane >> 3, rc = lane & 7;
    // the token ids of the rows this thread updates and of the rows of V it stages, looked up together and
    // before anything else is requested
    constexpr int c8 = KS * 4;  // staged chunks (8 ranks) per token
    static_assert(LORA_TILE_TOKENS * c8 == 256 * KS, "a thread stages KS pieces");
    int rows[4 + KS], toks[4 + KS];
#pragma unroll
    for (int i = 0; i < 4; ++i) rows[i] = 32 * th + 8 * i + rt;
#pragma unroll
    for (int i = 0; i < KS; ++i) rows[4 + i] = (tid + 256 * i) / c8;
    tile_tokens(a, it, rows, toks);
    size_t yoff[4];
    bool yok[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        yok[i] = rows[i] < it.n_tok;
        yoff[i] = (size_t)toks[i] * a.h_out + rc * 8;
    }
    const bool half_live = 32 * th < it.n_tok;
    const int col0 = col_run * n_pass * 128 + 64 * ch;

    // base_out of pass `cp`.  Read once and written once, both as streaming accesses: the rows then leave the caches
    // as they are written instead of lying there dirty until the next kernel's loads push them out (measured on the
    // kernels that follow: the tile shrink of the next projection or layer 93 -> 79 us on the mixed configuration,
    // 19.9 -> 17.3 us on the prefill one, for 0.6 us more in this kernel; either hint alone changes nothing)
    auto load_y = [&](int cp, uint4(&d)[4]) {
        const int nw0 = min(col0 + cp * 128, a.h_out - 64);
        typedef unsigned u32x4_nt __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const u32x4_nt t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt *>(y + yoff[i] + nw0));
            d[i] = make_uint4(t[0], t[1], t[2], t[3]);
        }
    };
    // Bp operands of the pass starting at column nw0: block b = columns nw0 + 16b .. +15, k step ks
    const __bf16 *bg[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) bg[ks] = Bp + ((size_t)min(4 * ks + g, rs8 - 1) * a.h_out + m) * 8;
    auto load_b = [&](int nw0, uint4(&d)[KS][4]) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int b = 0; b < 4; ++b) d[ks][b] = *reinterpret_cast<const uint4 *>(bg[ks] + (size_t)(nw0 + 16 * b) * 8);
    };

    uint4 yr[2][4];
    uint4 br[KS][4];

    // stage s.V (written as bf16 by the shrink or the reduce): vs[token][rank].  A thread's KS pieces (8 ranks of one
    // token each) are all requested before the first is used: taken one after the other, each with its own trip to
    // memory, the staging took 4.6 us (rank 16) to 8.2 us (rank 128) of a block's 17 to 21 us on the prefill
    // configuration.  V is requested first
    // and the first pass's base_out and Bp behind it (loads complete in the order of their requests): those are
    // on their way while V is staged.
    {
        const uint4 *vr[KS];
        bool ok[KS];
#pragma unroll
        for (int i = 0; i < KS; ++i) {
            const int idx = tid + 256 * i, ti = idx / c8, j8 = idx - ti * c8;
            ok[i] = ti < it.n_tok;
            vr[i] = reinterpret_cast<const uint4 *>(reinterpret_cast<const __bf16 *>(a.v) + (size_t)toks[4 + i] * (2 * a.v_stride) + j8 * 8);
        }
        uint4 pc[KS];
#pragma unroll
        for (int i = 0; i < KS; ++i) pc[i] = vr[i][0];
        __builtin_amdgcn_sched_barrier(0);  // keep the scheduler from trading loads in flight for registers
        load_y(0, yr[0]);
        load_b(min(col0, a.h_out - 64), br);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < KS; ++i) {
            const int idx = tid + 256 * i, ti = idx / c8, j8 = idx - ti * c8;
            const bf16x8 f = __builtin_bit_cast(bf16x8, pc[i]);
            bf16x8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (ok[i] && j8 * 8 + e < it.rank) ? f[e] : (__bf16)0.f;  // entries past the rank were never written
            *reinterpret_cast<bf16x8 *>(&vs[ti * VS_ROW + j8 * 16]) = o;
        }
    }
    __syncthreads();

    if (!half_live) return;  // this token half is empty (no barrier follows)
    unsigned char *my_cs = cs[w];

    // one pass of 128 columns; PAR = cp % 2 is a compile-time constant so that the base_out double
    // buffer stays in registers
    auto pass = [&](auto par_tag, int cp) {
        constexpr int PAR = decltype(par_tag)::value;
        const int nw0 = col0 + cp * 128;
        load_y(cp + 1, yr[PAR ^ 1]);  // next pass's base_out, ahead of this pass's products

        floatx4 acc[4][2];
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) acc[b][tb] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const bf16x8 aop = __builtin_bit_cast(bf16x8, br[ks][b]);
                const bf16x8 b0 = *reinterpret_cast<const bf16x8 *>(&vs[(32 * th + m) * VS_ROW + (4 * ks + g) * 16]);
                const bf16x8 b1 = *reinterpret_cast<const bf16x8 *>(&vs[(32 * th + 16 + m) * VS_ROW + (4 * ks + g) * 16]);
                acc[b][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop, b0, acc[b][0], 0, 0, 0);
                acc[b][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop, b1, acc[b][1], 0, 0, 0);
            }
        load_b(min(nw0 + 128, a.h_out - 64), br);  // next pass's Bp, into the registers just used

        // park the products: lane (g, m) holds, for block b and token block tb, columns 16b + 4g .. +3 of token 16tb + m
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
                *reinterpret_cast<floatx4 *>(&my_cs[(16 * tb + m) * CS_ROW + (16 * b + 4 * g) * 4]) = acc[b][tb];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // a wavefront's LDS operations execute in order
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float4 p0 = *reinterpret_cast<const float4 *>(&my_cs[(8 * i + rt) * CS_ROW + rc * 32]);
            const float4 p1 = *reinterpret_cast<const float4 *>(&my_cs[(8 * i + rt) * CS_ROW + rc * 32 + 16]);
            float f[8];
            Chunk<__bf16> c;
            c.v = yr[PAR][i];
            unpack_chunk(c, f);
            bf16x8 o;
            o[0] = (__bf16)(f[0] + p0.x); o[1] = (__bf16)(f[1] + p0.y); o[2] = (__bf16)(f[2] + p0.z); o[3] = (__bf16)(f[3] + p0.w);
            o[4] = (__bf16)(f[4] + p1.x); o[5] = (__bf16)(f[5] + p1.y); o[6] = (__bf16)(f[6] + p1.z); o[7] = (__bf16)(f[7] + p1.w);
            if (yok[i]) __builtin_nontemporal_store(o, reinterpret_cast<bf16x8 *>(y + yoff[i] + nw0));
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();  // the next pass overwrites the parked products
    };
    // columns past h_out: this wavefront's share of the block ends (the loads ahead were clamped)
    const int my_pass = min(n_pass, (a.h_out - col0 + 127) / 128);
    for (int cp = 0; cp < my_pass; cp += 2) {
        pass(std::integral_constant<int, 0>{}, cp);
        if (cp + 1 < my_pass) pass(std::integral_constant<int, 1>{}, cp + 1);
    }
}

// Blocks -> (tile, column run).  Block b runs on XCD b % 8; the blocks are numbered so that a column run -- the same
// columns of every tile -- always falls on the same XCD (or the same two or four), and a prompt's Bp is fetched
// from memory by one XCD per column run instead of by all eight (with the tiles as the fast index the prefill
// expand fetched 147 MB for 101 MB).  The column runs go in groups of eight: within a group block
// (tile * 8 + run % 8) works on that tile and run; what is left over after the whole groups forms a last group of
// 1, 2, 4 or 8 runs (the next power of two: at most a twelfth of a launch's blocks are padding, which return at once --
// padding every launch to a multiple of 8 runs cost the two 11-run launches of the mixed configuration 29 us each).
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void mfma_expand_kernel(ApplyArgs a, const DevItem *__restrict__ tiles, int n_tiles,
                                                                                                        int n_pass, int n_runs, int last_width)
{
    __shared__ __attribute__((aligned(16))) unsigned char vs[LORA_TILE_TOKENS * VS_ROW];
    __shared__ __attribute__((aligned(16))) unsigned char cs[4][32 * CS_ROW];
    const int whole = (n_runs >> 3) * n_tiles * 8;  // blocks of the groups of eight
    int tile, col_run;
    if ((int)blockIdx.x < whole) {
        const int grp = (int)blockIdx.x / (n_tiles * 8), r = (int)blockIdx.x - grp * n_tiles * 8;
        tile = r >> 3;
        col_run = 8 * grp + (r & 7);
    } else {
        const int r = (int)blockIdx.x - whole;
        tile = r / last_width;
        col_run = (n_runs & ~7) + (r - tile * last_width);
        if (col_run >= n_runs) return;  // padding
    }
    const DevItem it = tiles[tile];
    switch ((it.rank + 31) >> 5) {
    case 1: mfma_expand_body<1>(a, it, col_run, n_pass, vs, cs); break;
    case 2: mfma_expand_body<2>(a, it, col_run, n_pass, vs, cs); break;
    case 3: mfma_expand_body<3>(a, it, col_run, n_pass, vs, cs); break;
    default: mfma_expand_body<4>(a, it, col_run, n_pass, vs, cs); break;
    }
}

// k ranges are multiples of the 128-element stage.
hipError_t launch_mfma_shrink(const ApplyArgs &a, const ShrinkProjs &ps, const DevItem *tiles, int n_tiles, hipStream_t st,
                              const KernelTimer *tm)
{
    if (n_tiles <= 0 || ps.n <= 0 || ps.n_runs <= 0) return hipSuccess;
    if (ps.n_runs % 8 != 0 || ps.quanta < 1) return hipErrorInvalidValue;
    const int runs_per_xcd = ps.n_runs / 8;
    launch_k(tm, LORA_K_MFMA_SHRINK, mfma_shrink_kernel, dim3(ps.n_runs * ps.n), dim3(256), st, ps.cuts, tiles, runs_per_xcd, ps.n,
             ps.quanta, n_tiles, a, ps);
    if (ps.any_pieces)
        launch_k(tm, LORA_K_MFMA_REDUCE, mfma_reduce_kernel, dim3(n_tiles * 8, ps.n), dim3(256), st, a, ps, tiles);
    return hipGetLastError();
}

hipError_t launch_mfma_expand(const ApplyArgs &a, const DevItem *tiles, int n_tiles, hipStream_t st, const KernelTimer *tm)
{
    if (n_tiles <= 0) return hipSuccess;
    // the widest column run per block that still gives 512 blocks (two per CU), else the narrowest
    int cols = 1024;
    while (cols > 256 && (int64_t)n_tiles * ((a.h_out + cols - 1) / cols) < 512) cols >>= 1;
    const int n_runs = (a.h_out + cols - 1) / cols;
    int last_width = 0;  // of the last, partial group of column runs: the next power of two
    if (n_runs & 7) {
        last_width = 1;
        while (last_width < (n_runs & 7)) last_width <<= 1;
    }
    launch_k(tm, LORA_K_MFMA_EXPAND, mfma_expand_kernel, dim3(n_tiles * ((n_runs & ~7) + last_width)), dim3(256), st, a, tiles, n_tiles,
             cols / 128, n_runs, last_width);
    return hipGetLastError();
}

}  // namespace lora
