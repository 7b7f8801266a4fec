// GEMV path of the batched LoRA apply for gfx950: tokens whose slot has only a few tokens in
// the batch (decode requests, short prompts).  Both phases are bandwidth-bound streams of
// the slot's slab.  A work item is a batch of up to 4 tokens of one slot; every load an item
// needs -- slab, activations, intermediate -- is issued before the first one is used, so an
// item costs one trip to memory, and the batches of a popular slot run side by side (its slab
// then comes out of L2 for all but the first).
//
//   shrink:  v[t][j] = sum_k x[t][k] * A[k][j]        a block owns 4 rank rows of At, its wavefronts split k
//   expand:  y[t][n] += s * sum_j v[t][j] * B[j][n]   a wavefront owns a run of output columns of Bp (16 KB of it)
//
// One launch serves every projection of a group that reads the same activations (q, k, v; gate,
// up): block and unit numbers map to (projection, item).  The two phases run as one launch or as
// two.  In one launch the expand wavefronts fetch their part of Bp and base_out while the shrink
// blocks are still working and then pick up the intermediate, which travels as 64-bit words
// {launch number, payload}, written and read with device-scope atomic accesses (which go past the
// per-XCD L2s, not coherent with each other): a reader polls the words it needs until all carry
// the number of this launch, so there are no counters, no fences and no resets, and the hand-over
// costs one store and one load latency.  Payload: for bf16 two values s.v[j], s.v[j+1] rounded to
// bf16 (the expand product runs on the matrix cores, which take bf16 operands anyway; word
// tok * 64 + j / 2); for fp32 one value v[j] (word tok * 128 + j).  As two launches the words are
// written and read the same way, without the number.
//
// What sets the pace of a launch this small is the length of each wavefront's own path -- its
// dependent trips to memory and the number of instructions between them -- not the bytes: so
// addresses are a scalar base plus one 32-bit lane offset, sums over the wavefront fold through
// lane swaps and DPP instead of LDS permutes, and the expand of every rank runs as 16 matrix-core
// products per 16 KB of Bp (small ranks fill the product's k dimension with several column groups).
//
// (paper section 3.1: the two adapter products and the aggregation into the base output.)
#include <algorithm>

#include "lora_device.h"

namespace lora {

constexpr int TB = GEMV_BATCH;
static_assert(TB == 4 && GEMV_SHRINK_ROWS == 4, "the lane mappings below are written for batches of 4 tokens and items of 4 rows");
constexpr int WAIT_SPINS = 1 << 16;

template <typename E> constexpr int words_per_token() { return sizeof(E) == 2 ? 64 : 128; }

// 16 bytes of a slab: read once per launch (by the batches of one slot at about the same time), so marked
// as streaming -- they then do not push the work items and the kernel's own code out of L2 (-4 % on the
// decode configuration)
typedef unsigned gv_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_slab16(const char *p)
{
    const gv_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const gv_u32x4 *>(p));
    return make_uint4(v[0], v[1], v[2], v[3]);
}

// A work item as a wavefront holds it: every field the same in all lanes and said to be so, so that the
// fields and the addresses built from them stay in scalar registers; the tokens as four named members
// (an array indexed by a lane's token number would be kept in scratch memory).
struct ItemU {
    int tok0, tok1, tok2, tok3, row, rank, a;
    float alpha;
    __device__ __forceinline__ int tok(int t) const { return t == 0 ? tok0 : (t == 1 ? tok1 : (t == 2 ? tok2 : tok3)); }  // t constant or per lane
    __device__ __forceinline__ int n_tok() const { return 1 + (tok1 >= 0) + (tok2 >= 0) + (tok3 >= 0); }  // tokens fill the batch from the front
};
__device__ __forceinline__ ItemU load_item(const GemvItem *p)
{
    const int4 lo = *reinterpret_cast<const int4 *>(p), hi = *(reinterpret_cast<const int4 *>(p) + 1);
    ItemU u;
    u.tok0 = __builtin_amdgcn_readfirstlane(lo.x);
    u.tok1 = __builtin_amdgcn_readfirstlane(lo.y);
    u.tok2 = __builtin_amdgcn_readfirstlane(lo.z);
    u.tok3 = __builtin_amdgcn_readfirstlane(lo.w);
    u.row = __builtin_amdgcn_readfirstlane(hi.x);
    u.rank = __builtin_amdgcn_readfirstlane(hi.y);
    u.a = __builtin_amdgcn_readfirstlane(hi.z);
    u.alpha = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(hi.w));
    return u;
}
__device__ __forceinline__ GemvItem as_item(const ItemU &u)  // for the routines shared with the host
{
    GemvItem it;
    it.tok[0] = u.tok0, it.tok[1] = u.tok1, it.tok[2] = u.tok2, it.tok[3] = u.tok3;
    it.row = u.row, it.rank = u.rank, it.a = u.a, it.alpha = u.alpha;
    return it;
}

__device__ __forceinline__ void put_word(unsigned long long *p, uint32_t epoch, uint32_t payload)
{
    __hip_atomic_store(p, ((unsigned long long)epoch << 32) | payload, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One word per token of the batch and lane (word `lane` of the token's row; `need` says which lanes'
// words exist).  One launch: polls until every needed word of the wavefront carries this launch's
// number; bounded -- a wavefront that gives up raises the fault flag and does no work.
__device__ __forceinline__ bool fetch_words(const GemvArgs &a, const unsigned long long *const (&p)[TB], bool need, int nt,
                                            uint32_t (&out)[TB])
{
    if (a.epoch == 0) {
#pragma unroll
        for (int t = 0; t < TB; ++t) out[t] = (uint32_t)__hip_atomic_load(p[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return true;
    }
    // Polls travel the same way as the slabs, past the caches: only the words that are waited for are asked for (the
    // batch's own tokens -- nt is the same for the wavefront -- and the lanes below the stored rank), and a failed
    // poll is followed by a short sleep.  (With all four token slots and all 64 lanes polled back to back the decode
    // layer took 10.4 us instead of 9.65.)
    // The first poll goes out when the loads requested before it (the unit's Bp and base_out) are in: its answer would
    // come back behind them anyway, and asked for earlier it is nearly always a miss (decode layer 9.6 -> 9.45 us).
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    for (int spin = 0; spin < WAIT_SPINS; ++spin) {
        unsigned long long w[TB];
#pragma unroll
        for (int t = 0; t < TB; ++t) w[t] = (t < nt && need) ? __hip_atomic_load(p[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0ull;
        bool ok = true;
#pragma unroll
        for (int t = 0; t < TB; ++t) ok = ok && (!need || t >= nt || (uint32_t)(w[t] >> 32) == a.epoch);
        if (__all(ok)) {
#pragma unroll
            for (int t = 0; t < TB; ++t) out[t] = (uint32_t)w[t];
            return true;
        }
        __builtin_amdgcn_s_sleep(8);
    }
    if ((threadIdx.x & 63) == 0) __hip_atomic_store(a.fault, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);  // pinned host memory
    return false;
}

// ---------------------------------------------------------------------------------------
// shrink.  A work item names 4 stored rank rows of a slot and up to 4 tokens, and is worked on by
// one block of W wavefronts that split k: the rows are cut into runs of 64 chunks (8 elements each)
// and wavefront kp covers runs kp and kp + W of a pass (fp32: one run), so a lane loads 2 chunks of
// each of the 4 rows and the same 2 chunks of x of each token -- x is fetched once per item, not once
// per row -- all before the first use, then forms the 4 x NT dot products.  Rows longer than W * 2 runs
// take more passes.  Few registers and 8 KB of slab per wavefront in flight: many wavefronts fit a CU
// and their memory phases overlap.  Sums are folded over the 64 lanes and added over the W wavefronts
// through LDS.  NT = 1, 2 or 4 (a batch of 3 runs as one of 4 with its first token repeated).
// ---------------------------------------------------------------------------------------
template <typename E, int NT>
__device__ __forceinline__ void gemv_shrink_item(const GemvArgs &a, const GemvProj &pj, const ItemU it, int nt, float (*red)[16])
{
    constexpr int U = sizeof(E) == 2 ? 2 : 1;  // runs per wavefront and pass (fp32 chunks take twice the registers)
    constexpr int NV = 4 * NT;                 // values folded; value 4t + r is row r of token t
    const int lane = threadIdx.x & 63;
    const int kp = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), W = blockDim.x >> 6;
    const int n_chunks = a.h_in >> 3;
    const size_t row_b = (size_t)a.h_in * sizeof(E);
    int j0, n_rows;
    gemv_shrink_rows(as_item(it), j0, n_rows);
    const char *arow[4], *xrow[NT];
    const char *slab = pj.proj_base + (int64_t)it.row * pj.row_bytes;
#pragma unroll
    for (int r = 0; r < 4; ++r) arow[r] = slab + (size_t)(j0 + r) * row_b;
#pragma unroll
    for (int t = 0; t < NT; ++t) xrow[t] = static_cast<const char *>(a.x) + (size_t)(t < nt ? it.tok(t) : it.tok0) * row_b;

    float acc[4][NT];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[r][t] = 0.f;

    // Loads are unconditional (chunks past the row end clamped to its last, results masked), so that
    // all of them are issued back to back and waited for once.
    for (int c0 = 0; c0 < n_chunks; c0 += W * 64 * U) {
        Chunk<E> xv[NT][U], av[4][U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t off = (uint32_t)min(c0 + (u * W + kp) * 64 + lane, n_chunks - 1) * (uint32_t)(8 * sizeof(E));
#pragma unroll
            for (int t = 0; t < NT; ++t) xv[t][u] = *reinterpret_cast<const Chunk<E> *>(xrow[t] + off);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if constexpr (sizeof(E) == 2) av[r][u].v = load_slab16(arow[r] + off);
                else av[r][u] = *reinterpret_cast<const Chunk<E> *>(arow[r] + off);
            }
        }
        __builtin_amdgcn_sched_barrier(0);  // keep the scheduler from trading loads in flight for registers
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool ok = c0 + (u * W + kp) * 64 + lane < n_chunks;  // clamped lanes do not count: their x is zeroed
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const Chunk<E> xz = ok ? xv[t][u] : zero_chunk<E>();
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[r][t] = dot_chunk_acc(acc[r][t], av[r][u], xz);
            }
        }
    }
    float sum[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) sum[i] = acc[i & 3][i >> 2];
    wave_fold(sum);  // value i now on the lanes i * (64 / NV) ..
    if (lane % (64 / NV) == 0) red[kp][lane / (64 / NV)] = sum[0];
    __syncthreads();
    if (kp != 0) return;
    float val = 0.f;
    for (int q = 0; q < W; ++q) val += red[q][lane & 15];
    const int t = (lane >> 2) & 3, r = lane & 3;
    const int tok = it.tok(t);
    if constexpr (sizeof(E) == 2) {
        // two rows to a word, scaled and rounded to bf16: what the expand product takes
        const float s = a.scale * it.alpha;
        const float nxt = __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, val), 0xB1, 0xF, 0xF, true));  // lane ^ 1
        typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
        bf16x2_t pr;
        pr[0] = (__bf16)(s * val);
        pr[1] = (__bf16)(s * nxt);
        if (lane < NV && t < nt && (r & 1) == 0)
            put_word(pj.vw + (size_t)tok * 64 + ((j0 + r) >> 1), a.epoch, __builtin_bit_cast(uint32_t, pr));
    } else {
        if (lane < NV && t < nt) put_word(pj.vw + (size_t)tok * 128 + j0 + r, a.epoch, __float_as_uint(val));
    }
}

// ---------------------------------------------------------------------------------------
// expand, bf16.  One wavefront per unit: a token batch x 16 KB of Bp = the columns [c0, c1) of
// gemv_expand_width(rank) (less at the ragged end of a projection).  The per-column dot products
// over the rank go to v_mfma_f32_16x16x32_bf16 with the product formed transposed,
// D[column][n] = A[column][k] . B[k][n]:
//   A: lane (m = lane % 16, g = lane / 16) supplies k = 8g .. 8g+7 of row m -- one 16-byte chunk of Bp
//      exactly as it lies in the pool (8 ranks of one column);
//   B: lane (n = lane % 16, g) supplies k = 8g .. 8g+7 of column n -- s.v as bf16 out of LDS;
//   D: lane (n, r = lane / 16) holds rows 4r .. 4r+3 of column n -- 4 consecutive output columns of one token.
// From 32 stored ranks up (G = 1) a product covers 16 columns and 32 ranks (KS products per 16
// columns for up to 128 ranks), n = token.  Below, the 32 k of a product hold G = 2 or 4 column groups
// side by side (16 or 8 ranks each) and B is block diagonal, n = token + 4 * group: k slot g belongs to
// group g / (4 / G) and meets s.v only in the columns n of its own group, zeros elsewhere.  So a product
// always consumes a full 1 KB of Bp, a unit is at most 16 products, and the output lanes of a token
// form whole 32- to 128-byte runs of base_out.
// ---------------------------------------------------------------------------------------
typedef __bf16 gv_bf16x8 __attribute__((ext_vector_type(8)));
typedef float gv_floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 gv_bf16x4 __attribute__((ext_vector_type(4)));

template <int G, int KS>
__device__ __forceinline__ void gemv_expand_mfma(const GemvArgs &a, const GemvProj &pj, const ItemU it, int nt, int c0, int c1,
                                                 uint32_t *vb /* this wavefront's LDS: [TB][64] words */)
{
    constexpr int NQ = 16 / KS;   // column spans (one accumulator each) of a whole unit
    constexpr int SPAN = 16 * G;  // columns per span
    const int lane = threadIdx.x & 63, m = lane & 15, g = lane >> 4;
    const int rs = rank_storage(it.rank), rs8 = rs >> 3;
    const int n_q = (c1 - c0) / SPAN;  // spans of this unit (widths are multiples of 64)
    const char *Bp = pj.proj_base + (int64_t)it.row * pj.row_bytes + (size_t)rs * a.h_in * 2 + (size_t)c0 * 16;

    // lane part of the Bp addresses: (granule * h_out + column within the span) * 16 bytes
    uint32_t boff[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        if constexpr (G == 4) boff[ks] = (uint32_t)lane * 16u;                                                 // group g, granule 0
        else if constexpr (G == 2) boff[ks] = ((uint32_t)(g & 1) * pj.h_out + 16u * (g >> 1) + m) * 16u;       // group g / 2, granule g % 2
        else boff[ks] = ((uint32_t)min(4 * ks + g, rs8 - 1) * pj.h_out + m) * 16u;  // granules past the stored rank repeat the last (they meet zeros)
    }
    // all loads up front, unconditional: spans past the unit repeat its first
    uint4 br[NQ][KS];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const char *bq = Bp + (q < n_q ? q * SPAN * 16 : 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) br[q][ks] = load_slab16(bq + boff[ks]);
    }
    // base_out: lane (n, r) updates columns 16 * group + 4r .. +3 of the span for token n % 4
    const int t = m & 3, gq = m >> 2;
    const bool live = gq < G && t < nt;
    const int tok_l = live ? it.tok(t) : it.tok0;
    const uint32_t yoff = (uint32_t)tok_l * pj.h_out + (live ? 16 * gq : 0) + 4 * g;  // elements from column c0 of row 0
    const char *ybase = static_cast<const char *>(pj.y) + (size_t)c0 * 2;
    uint2 yv[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) yv[q] = *reinterpret_cast<const uint2 *>(ybase + (q < n_q ? q * SPAN * 2 : 0) + yoff * 2u);

    // the intermediate: word `lane` of every token's row holds ranks 2 lane, 2 lane + 1
    const unsigned long long *vp[TB];
#pragma unroll
    for (int tt = 0; tt < TB; ++tt) vp[tt] = pj.vw + (size_t)(tt < nt ? it.tok(tt) : it.tok0) * 64 + lane;
    uint32_t vword[TB];
    if (!fetch_words(a, vp, 2 * lane < rs, nt, vword)) return;
#pragma unroll
    for (int tt = 0; tt < TB; ++tt) vb[tt * 64 + lane] = (tt < nt && 2 * lane < rs) ? vword[tt] : 0u;
    // only this wavefront reads what it wrote, and a wavefront's LDS operations execute in order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    gv_bf16x8 vop[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        int gran;
        bool mine;
        if constexpr (G == 4) gran = 0, mine = g == gq;
        else if constexpr (G == 2) gran = g & 1, mine = (g >> 1) == gq;
        else gran = 4 * ks + g, mine = gq == 0;
        const uint4 w = *reinterpret_cast<const uint4 *>(vb + t * 64 + 4 * gran);
        const uint4 z = make_uint4(0u, 0u, 0u, 0u);
        vop[ks] = __builtin_bit_cast(gv_bf16x8, mine ? w : z);
    }
    auto product = [&](int q) {
        gv_floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(gv_bf16x8, br[q][ks]), vop[ks], acc, 0, 0, 0);
        return acc;
    };
    if (pj.y32) {  // uniform
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const gv_floatx4 acc = product(q);
            if (live && q < n_q) *reinterpret_cast<gv_floatx4 *>(pj.y32 + (size_t)c0 + q * SPAN + yoff) = acc;
        }
        return;
    }
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const gv_floatx4 acc = product(q);
        const unsigned lo = yv[q].x, hi = yv[q].y;
        gv_bf16x4 o;
        o[0] = (__bf16)(__uint_as_float(lo << 16) + acc[0]);
        o[1] = (__bf16)(__uint_as_float(lo & 0xffff0000u) + acc[1]);
        o[2] = (__bf16)(__uint_as_float(hi << 16) + acc[2]);
        o[3] = (__bf16)(__uint_as_float(hi & 0xffff0000u) + acc[3]);
        if (live && q < n_q) *reinterpret_cast<gv_bf16x4 *>(const_cast<char *>(ybase) + q * SPAN * 2 + yoff * 2u) = o;
    }
}

// expand, fp32 (the small full-precision configuration): granule loop on the vector ALUs, s.v of the
// item's tokens staged in this wavefront's LDS rows.
__device__ __forceinline__ void gemv_expand_f32(const GemvArgs &a, const GemvProj &pj, const ItemU it, int nt, int c0, int c1,
                                                float *vs /* [TB][128] */)
{
    const int lane = threadIdx.x & 63;
    const int rs = rank_storage(it.rank), rs8 = rs >> 3;
    const float s = a.scale * it.alpha;
    const float *Bp = reinterpret_cast<const float *>(pj.proj_base + (int64_t)it.row * pj.row_bytes) + (size_t)rs * a.h_in;
    float *y = static_cast<float *>(pj.y);
    for (int half = 0; half < 2; ++half) {
        const int j = half * 64 + lane;
        const unsigned long long *vp[TB];
#pragma unroll
        for (int tt = 0; tt < TB; ++tt) vp[tt] = pj.vw + (size_t)(tt < nt ? it.tok(tt) : it.tok0) * 128 + j;
        uint32_t vword[TB] = {0u, 0u, 0u, 0u};
        if (half * 64 < rs) {  // uniform
            if (!fetch_words(a, vp, j < rs, nt, vword)) return;
        }
#pragma unroll
        for (int tt = 0; tt < TB; ++tt) vs[tt * 128 + j] = (half * 64 < rs && tt < nt && j < it.rank) ? s * __uint_as_float(vword[tt]) : 0.f;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    for (int n = c0 + lane; n < c1; n += 64) {
        float acc[TB];
#pragma unroll
        for (int tt = 0; tt < TB; ++tt) acc[tt] = 0.f;
        for (int j8 = 0; j8 < rs8; ++j8) {
            float bf[8];
            unpack_chunk(load_chunk(Bp + ((size_t)j8 * pj.h_out + n) * 8), bf);
#pragma unroll
            for (int tt = 0; tt < TB; ++tt)
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[tt] += vs[tt * 128 + j8 * 8 + i] * bf[i];
        }
#pragma unroll
        for (int tt = 0; tt < TB; ++tt) {
            if (tt < nt) {
                const size_t idx = (size_t)it.tok(tt) * pj.h_out + n;
                if (pj.y32) pj.y32[idx] = acc[tt];
                else y[idx] += acc[tt];
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// the kernel: blocks of 4 wavefronts.  Blocks [0, n_proj * n_gs) are the shrink blocks, one (item,
// projection) each; the rest hold 4 expand wavefronts each, one unit = (projection, item, super-chunk)
// per wavefront.  Shrink blocks come first in the grid and wait for nothing, so waiting expand
// wavefronts cannot starve them; waits are bounded all the same.
// ---------------------------------------------------------------------------------------
template <typename E>
__global__ __launch_bounds__(256) void gemv_kernel(const GemvItem *gs, const GemvItem *ge, uint32_t n_gs, uint32_t n_proj_phase, int32_t ue0,
                                                   int32_t ue1, int32_t ue2, int32_t ue3, uint32_t n_super_packed, uint32_t sm0, uint32_t sm1,
                                                   uint32_t sm2, uint32_t sm3, GemvArgs a)
{
    // (the scalars in front are the fields of GemvMap one by one: the leading arguments of a kernel arrive in
    // registers with the wavefront)
    __shared__ float red[4][16];
    __shared__ __attribute__((aligned(16))) uint32_t stage[4][sizeof(E) == 2 ? TB * 64 : TB * 128];
    const uint32_t n_proj = n_proj_phase & 0xffu, phase = n_proj_phase >> 8;
    const uint32_t n_shrink = phase == 2 ? 0u : n_proj * n_gs;
    if (blockIdx.x < n_shrink) {
        uint32_t item, proj;
        gemv_shrink_block(blockIdx.x, n_gs, n_proj, item, proj);
        const ItemU it = load_item(gs + item);
        const GemvProj pj = a.p[proj];
        const int nt = it.n_tok();
        if (nt == 1) gemv_shrink_item<E, 1>(a, pj, it, nt, red);  // uniform over the block
        else if (nt == 2) gemv_shrink_item<E, 2>(a, pj, it, nt, red);
        else gemv_shrink_item<E, 4>(a, pj, it, nt, red);
    } else {
        if (phase == 1) return;
        const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const uint32_t unit = (blockIdx.x - n_shrink) * 4 + w;
        const GemvMap m{gs, ge, n_gs, n_proj_phase, {ue0, ue1, ue2, ue3}, n_super_packed, {sm0, sm1, sm2, sm3}};
        if (unit >= (uint32_t)ue3) return;  // (entries past the group repeat its last)
        uint32_t proj, item, sc;
        gemv_expand_unit(unit, m, proj, item, sc);
        const ItemU it = load_item(ge + item);
        const GemvProj pj = a.p[proj];
        int c0, c1;
        gemv_expand_cols(as_item(it), (int)sc, pj.h_out, c0, c1);
        if (c0 >= c1) return;
        const int nt = it.n_tok();
        if constexpr (sizeof(E) == 2) {
            const int rs8 = rank_storage(it.rank) >> 3;  // uniform over the wavefront
            if (rs8 == 1) gemv_expand_mfma<4, 1>(a, pj, it, nt, c0, c1, stage[w]);
            else if (rs8 == 2) gemv_expand_mfma<2, 1>(a, pj, it, nt, c0, c1, stage[w]);
            else if (rs8 <= 4) gemv_expand_mfma<1, 1>(a, pj, it, nt, c0, c1, stage[w]);
            else if (rs8 <= 8) gemv_expand_mfma<1, 2>(a, pj, it, nt, c0, c1, stage[w]);
            else if (rs8 <= 12) gemv_expand_mfma<1, 3>(a, pj, it, nt, c0, c1, stage[w]);
            else gemv_expand_mfma<1, 4>(a, pj, it, nt, c0, c1, stage[w]);
        } else {
            gemv_expand_f32(a, pj, it, nt, c0, c1, reinterpret_cast<float *>(stage[w]));
        }
    }
}

// zeroes the hand-over words of the listed tokens: one block per token
template <typename E>
__global__ __launch_bounds__(64) void gemv_clear_kernel(unsigned long long *vw, const int32_t *__restrict__ toks)
{
    constexpr int WPT = words_per_token<E>();
    unsigned long long *row = vw + (size_t)toks[blockIdx.x] * WPT;
    for (int i = threadIdx.x; i < WPT; i += 64) row[i] = 0ull;
}

size_t gemv_handover_bytes(int dtype, int64_t max_tokens)
{
    return sizeof(unsigned long long) * (size_t)max_tokens * (dtype == LORA_BF16 ? words_per_token<__bf16>() : words_per_token<float>());
}

hipError_t launch_gemv_clear(int dtype, unsigned long long *vw, const int32_t *toks, int n, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    if (dtype == LORA_BF16) hipLaunchKernelGGL(gemv_clear_kernel<__bf16>, dim3(n), dim3(64), 0, st, vw, toks);
    else hipLaunchKernelGGL(gemv_clear_kernel<float>, dim3(n), dim3(64), 0, st, vw, toks);
    return hipGetLastError();
}

hipError_t launch_gemv(int dtype, const GemvMap &m, const GemvArgs &a, hipStream_t st, const KernelTimer *tm)
{
    const int n_proj = (int)(m.n_proj_phase & 0xffu);
    if (m.n_gs == 0 || a.n_ge <= 0 || n_proj <= 0) return hipSuccess;
    const int n_shrink = n_proj * (int)m.n_gs, n_expand = (m.unit_end[GEMV_MAX_PROJS - 1] + 3) / 4;
    auto go = [&](uint32_t phase, int blocks, int kind) {
        const uint32_t pp = (uint32_t)n_proj | (phase << 8);
        if (dtype == LORA_BF16)
            launch_k(tm, kind, gemv_kernel<__bf16>, dim3(blocks), dim3(256), st, m.gs, m.ge, m.n_gs, pp, m.unit_end[0], m.unit_end[1],
                     m.unit_end[2], m.unit_end[3], m.n_super_packed, m.super_magic[0], m.super_magic[1], m.super_magic[2], m.super_magic[3], a);
        else
            launch_k(tm, kind, gemv_kernel<float>, dim3(blocks), dim3(256), st, m.gs, m.ge, m.n_gs, pp, m.unit_end[0], m.unit_end[1],
                     m.unit_end[2], m.unit_end[3], m.n_super_packed, m.super_magic[0], m.super_magic[1], m.super_magic[2], m.super_magic[3], a);
    };
    if (a.epoch) {
        go(0u, n_shrink + n_expand, LORA_K_GEMV_FUSED);
    } else {
        go(1u, n_shrink, LORA_K_GEMV_SHRINK);
        go(2u, n_expand, LORA_K_GEMV_EXPAND);
    }
    return hipGetLastError();
}

}  // namespace lora
