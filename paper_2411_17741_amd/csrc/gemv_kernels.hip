// GEMV path of the batched LoRA apply for gfx950: tokens whose slot has only a few tokens in
// the batch (decode requests, short prompts).  Both phases are bandwidth-bound streams of
// the slot's slab.  A work item is a batch of up to 4 tokens of one slot; every load an item
// needs -- slab, activations, intermediate -- is issued before the first one is used, so an
// item costs one trip to memory, and the batches of a popular slot run side by side (its slab
// then comes out of L2 for all but the first).
//
//   shrink:  v[t][j] = sum_k x[t][k] * A[k][j]        wavefronts own (parts of) rank rows of At
//   expand:  y[t][n] += s * sum_j v[t][j] * B[j][n]   a wavefront owns a run of output columns of Bp
//
// The two phases run as two launches, or -- as an option -- as one (fused) launch, in which the
// expand wavefronts fetch their part of Bp and base_out while the shrink blocks are still working
// and then pick up the intermediate.  In the fused form every value of v travels as one 64-bit
// word {apply number, fp32 bits}, written and read with device-scope atomic accesses (which go
// past the per-XCD L2s, not coherent with each other): a reader polls the words it needs until
// all carry the number of this apply, so there are no counters, no fences and no resets, and the
// hand-over costs one store and one load latency.  (Not under stream capture: a graph would freeze
// the number.)
//
// (paper section 3.1: the two adapter products and the aggregation into the base output.)
#include <algorithm>

#include "lora_device.h"

namespace lora {

constexpr int TB = GEMV_BATCH;
constexpr int GEMV_DP_ROW = 256 + 4;  // floats per token row of an expand wavefront's LDS (widest unit, padded)

// How the two phases hand over v.
struct Handover {
    unsigned long long *vtag;  // nullptr: separate launches, the stream orders the phases, v is plain fp32
    uint32_t epoch;            // number of this apply; never 0, never reused while older words may remain
    int32_t *fault;
};

__device__ __forceinline__ void publish_v(const Handover &ho, size_t idx, float val)
{
    const unsigned long long w = ((unsigned long long)ho.epoch << 32) | __float_as_uint(val);
    __hip_atomic_store(ho.vtag + idx, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Polls N tagged words per lane until every needed one, over the whole wavefront, carries this
// apply's number.  Bounded: a wavefront that gives up raises the fault flag and does no work.
template <int N>
__device__ __forceinline__ bool fetch_v(const Handover &ho, const unsigned long long *const (&p)[N], const bool (&need)[N],
                                        float (&out)[N])
{
    for (int spin = 0; spin < (1 << 16); ++spin) {
        unsigned long long w[N];
#pragma unroll
        for (int i = 0; i < N; ++i) w[i] = __hip_atomic_load(p[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bool ok = true;
#pragma unroll
        for (int i = 0; i < N; ++i) ok = ok && (!need[i] || (uint32_t)(w[i] >> 32) == ho.epoch);
        if (__all(ok)) {
#pragma unroll
            for (int i = 0; i < N; ++i) out[i] = __uint_as_float((uint32_t)w[i]);
            return true;
        }
        __builtin_amdgcn_s_sleep(2);
    }
    if ((threadIdx.x & 63) == 0) __hip_atomic_store(ho.fault, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);  // pinned host memory
    return false;
}

// ---------------------------------------------------------------------------------------
// shrink.  A work item names up to 4 rank rows of a slot and up to 4 tokens, and is worked on
// by one block of W wavefronts that split k: the rows are cut into runs of 64 chunks (8
// elements each) and wavefront kp covers runs kp and kp + W, so a lane loads 2 chunks of each of
// the 4 rows and the same 2 chunks of x of each token (fp32: one run, one chunk) -- x is fetched once per item, not once
// per row -- all before the first use, then forms the 4 x NT dot products.  W is chosen by the
// launcher so that the whole row is covered in one pass (rows longer than 16 * 2 runs take
// more).  Few registers and 8 KB of slab per wavefront in flight: many wavefronts fit a CU and
// their memory phases overlap.  Sums are folded over the 64 lanes and added over the W
// wavefronts through LDS.
// ---------------------------------------------------------------------------------------
template <typename E> constexpr int shrink_u() { return sizeof(E) == 2 ? 2 : 1; }  // runs per wavefront and pass (fp32 chunks take twice the registers)
constexpr int SHRINK_MAX_W = 16;   // wavefronts per block

template <typename E, int NT>
__device__ __forceinline__ void gemv_shrink_partial(const ApplyArgs &a, const GemvItem &it, int kp, int W,
                                                    float (&sum)[4 * (NT == 3 ? 4 : NT)])
{
    constexpr int U = shrink_u<E>();
    const int lane = threadIdx.x & 63;
    int j0, n_rows;
    gemv_shrink_rows(it, j0, n_rows);
    const E *slab = reinterpret_cast<const E *>(a.proj_base + (int64_t)it.row * a.row_bytes);
    const E *arow[4], *xrow[NT];
#pragma unroll
    for (int r = 0; r < 4; ++r) arow[r] = slab + (size_t)(j0 + min(r, n_rows - 1)) * a.h_in;  // rows past the item repeat its last
#pragma unroll
    for (int t = 0; t < NT; ++t) xrow[t] = static_cast<const E *>(a.x) + (size_t)it.tok[t] * a.h_in;
    const int n_chunks = a.h_in >> 3;

    float acc[4][NT];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[r][t] = 0.f;

    // Loads are unconditional (chunks past the row end clamped to its last, results masked), so
    // that the compiler can issue all of them back to back and wait once.
    for (int c0 = 0; c0 < n_chunks; c0 += W * 64 * U) {
        Chunk<E> xv[NT][U], av[4][U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t c = (size_t)min(c0 + (u * W + kp) * 64 + lane, n_chunks - 1) * 8;
#pragma unroll
            for (int t = 0; t < NT; ++t) xv[t][u] = load_chunk(xrow[t] + c);
#pragma unroll
            for (int r = 0; r < 4; ++r) av[r][u] = load_chunk(arow[r] + c);
        }
        __builtin_amdgcn_sched_barrier(0);  // keep the scheduler from trading loads in flight for registers
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool ok = c0 + (u * W + kp) * 64 + lane < n_chunks;  // clamped lanes do not count
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const float d = dot_chunk_acc(0.f, av[r][u], xv[t][u]);
                    acc[r][t] += ok ? d : 0.f;
                }
        }
    }
    // value 4t + r; a batch of 3 tokens is folded as one of 4
#pragma unroll
    for (int i = 0; i < 4 * (NT == 3 ? 4 : NT); ++i) sum[i] = (i >> 2) < NT ? acc[i & 3][(i >> 2) < NT ? (i >> 2) : 0] : 0.f;
    wave_sum_fold(sum);
}

// `red`: [W][16] floats of LDS.  Every wavefront of the block passes the barrier once.
template <typename E, int NT>
__device__ __forceinline__ void gemv_shrink_item(const ApplyArgs &a, const GemvItem &it, const Handover &ho, float (*red)[16])
{
    constexpr int NV = 4 * (NT == 3 ? 4 : NT);  // values folded; value i is on the lanes i * (64 / NV) ..
    const int lane = threadIdx.x & 63, kp = threadIdx.x >> 6, W = blockDim.x >> 6;
    float sum[NV];
    gemv_shrink_partial<E, NT>(a, it, kp, W, sum);
    if (lane % (64 / NV) == 0) red[kp][lane / (64 / NV)] = sum[0];
    __syncthreads();
    if (kp != 0 || lane >= NV) return;
    float val = 0.f;
    for (int q = 0; q < W; ++q) val += red[q][lane];
    const int t = lane >> 2, r = lane & 3;
    int j0, n_rows;
    gemv_shrink_rows(it, j0, n_rows);
    if (t < NT && r < n_rows) {
        const int tok = t == 0 ? it.tok[0] : (t == 1 ? it.tok[1] : (t == 2 ? it.tok[2] : it.tok[3]));
        const size_t idx = (size_t)tok * a.v_stride + j0 + r;
        if (ho.vtag) publish_v(ho, idx, val);
        else a.v[idx] = val;
    }
}

template <typename E>
__device__ __forceinline__ void gemv_shrink_dispatch(const ApplyArgs &a, const GemvItem &it, const Handover &ho, float (*red)[16])
{
    const int nt = (it.tok[1] >= 0) + (it.tok[2] >= 0) + (it.tok[3] >= 0);  // tokens fill the batch from the front
    switch (nt) {  // uniform over the block
        case 0: gemv_shrink_item<E, 1>(a, it, ho, red); break;
        case 1: gemv_shrink_item<E, 2>(a, it, ho, red); break;
        case 2: gemv_shrink_item<E, 3>(a, it, ho, red); break;
        default: gemv_shrink_item<E, 4>(a, it, ho, red); break;
    }
}

// v of the item's tokens, lane l holding entries l and (TWO) l + 64 of every row; entries past the
// rank and rows of unused tokens come back as anything.  False if a fused wait gave up.
template <bool TWO>
__device__ __forceinline__ bool fetch_v_rows(const ApplyArgs &a, const GemvItem &it, const Handover &ho, float (&vlo)[TB],
                                             float (&vhi)[TB])
{
    const int lane = threadIdx.x & 63;
    if (ho.vtag) {
        const unsigned long long *vp[2 * TB];
        bool need[2 * TB];
        float got[2 * TB];
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            const int tok = it.tok[t] >= 0 ? it.tok[t] : it.tok[0];
            vp[2 * t] = ho.vtag + (size_t)tok * a.v_stride + lane;  // rows are at least 128 entries long
            vp[2 * t + 1] = vp[2 * t] + (TWO ? 64 : 0);
            need[2 * t] = it.tok[t] >= 0 && lane < it.rank;
            need[2 * t + 1] = TWO && it.tok[t] >= 0 && lane + 64 < it.rank;
        }
        if (!fetch_v(ho, vp, need, got)) return false;
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            vlo[t] = got[2 * t];
            vhi[t] = got[2 * t + 1];
        }
    } else {
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            const int tok = it.tok[t] >= 0 ? it.tok[t] : it.tok[0];
            const float *vr = a.v + (size_t)tok * a.v_stride;  // rows are at least 128 floats long
            vlo[t] = vr[lane];
            vhi[t] = TWO ? vr[lane + 64] : 0.f;
        }
    }
    return true;
}

// ---------------------------------------------------------------------------------------
// expand, ranks whose storage is 8, 16, 32, 64 or 128 rows (RS8 = 1, 2, 4, 8, 16 granules).
// One wavefront per unit; a lane owns P = 16/RS8 output columns (n = c0 + lane + 64p) and
// loads all of its 16 chunks of Bp and the base_out values it will update up front, then the
// v of the item's tokens (one value per lane, broadcast with readlane when used).
// ---------------------------------------------------------------------------------------
template <typename E, int RS8>
__device__ __forceinline__ void gemv_expand_body(const ApplyArgs &a, const GemvItem &it, int c0, int c1, const E *Bp,
                                                 const Handover &ho)
{
    constexpr int P = 16 / RS8;
    const int lane = threadIdx.x & 63;
    const float s = a.scale * it.alpha;
    E *y = static_cast<E *>(a.y);

    // Loads are unconditional (columns and tokens clamped to valid ones, results discarded), so
    // that all of them are issued back to back; stores come after all the arithmetic.
    Chunk<E> b[P][RS8];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int n = c0 + lane + 64 * p;
        const int ns = n < c1 ? n : c0 + lane;
#pragma unroll
        for (int j8 = 0; j8 < RS8; ++j8) b[p][j8] = load_chunk(Bp + ((size_t)j8 * a.h_out + ns) * 8);
    }
    E yv[TB][P];
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        const int tok = it.tok[t] >= 0 ? it.tok[t] : it.tok[0];
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int n = c0 + lane + 64 * p;
            yv[t][p] = y[(size_t)tok * a.h_out + (n < c1 ? n : c0 + lane)];
        }
    }
    float vlo[TB], vhi[TB];
    if (!fetch_v_rows<(RS8 > 8)>(a, it, ho, vlo, vhi)) return;
    float acc[TB][P];
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        if (lane >= it.rank) vlo[t] = 0.f;  // what lies beyond the rank was never written
        if (lane + 64 >= it.rank) vhi[t] = 0.f;
#pragma unroll
        for (int p = 0; p < P; ++p) acc[t][p] = 0.f;
    }
#pragma unroll
    for (int j8 = 0; j8 < RS8; ++j8) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            float bf[8];
            unpack_chunk(b[p][j8], bf);
#pragma unroll
            for (int t = 0; t < TB; ++t) {
                if (it.tok[t] >= 0) {  // uniform
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int jj = j8 * 8 + i;
                        const float vj = __builtin_bit_cast(
                            float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, jj < 64 ? vlo[t] : vhi[t]), jj & 63));
                        acc[t][p] += vj * bf[i];
                    }
                }
            }
        }
    }
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        if (it.tok[t] >= 0) {
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const int n = c0 + lane + 64 * p;
                if (n < c1) {
                    if (a.y32) a.y32[(size_t)it.tok[t] * a.h_out + n] = s * acc[t][p];
                    else y[(size_t)it.tok[t] * a.h_out + n] = from_float<E>(to_float(yv[t][p]) + s * acc[t][p]);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// expand of bf16 slabs from 32 stored ranks up: the per-column dot products over the rank go to
// the matrix cores, which takes the arithmetic out of the vector ALUs (on those the unit costs
// about a thousand instructions, and the instruction stream, not memory, sets the pace).  The
// product is formed transposed, D[column][token] = Bp[column][rank] . (s v)[rank][token], with
// v_mfma_f32_16x16x32_bf16: the A operand of column block b and k step ks is one 16-byte chunk
// of Bp per lane (column c0 + 16b + lane%16, granule 4ks + lane/16), loaded as it lies; the B
// operand is s.v as bf16 out of this wavefront's LDS rows (token lane%16, of which the first 4
// exist); of the result a lane with lane%16 < 4 holds 4 consecutive columns of its token.
// KS = k steps (32 ranks each), NCB = column blocks of a full unit.
// ---------------------------------------------------------------------------------------
typedef __bf16 gv_bf16x8 __attribute__((ext_vector_type(8)));
typedef float gv_floatx4 __attribute__((ext_vector_type(4)));

template <int KS, int NCB>
__device__ __forceinline__ void gemv_expand_mfma(const ApplyArgs &a, const GemvItem &it, int c0, int c1, const __bf16 *Bp,
                                                 const Handover &ho, float (*vs)[GEMV_DP_ROW])
{
    const int lane = threadIdx.x & 63, m = lane & 15, g = lane >> 4;
    const int rs8 = rank_storage(it.rank) >> 3;
    const float s = a.scale * it.alpha;
    __bf16 *y = static_cast<__bf16 *>(a.y);
    const int n_cb = (c1 - c0) >> 4;  // column blocks of this unit (the last unit of a super-chunk may be cut)

    // all loads up front, unconditional: blocks past the unit repeat its first, granules past the
    // stored rank repeat the last (they meet zeros of v)
    uint4 br[NCB][KS];
#pragma unroll
    for (int b = 0; b < NCB; ++b) {
        const int cb = c0 + (b < n_cb ? 16 * b : 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            br[b][ks] = *reinterpret_cast<const uint4 *>(Bp + ((size_t)min(4 * ks + g, rs8 - 1) * a.h_out + cb + m) * 8);
    }
    // base_out is read and written with whole 128-byte lines: lane l covers, in line i of the
    // unit, the 4 columns 64i + 4(l%16) .. of token l/16
    const int tq = lane >> 4, q = lane & 15;
    const int tok_q = tq == 0 ? it.tok[0] : (tq == 1 ? it.tok[1] : (tq == 2 ? it.tok[2] : it.tok[3]));
    __bf16 *yrow = y + (size_t)(tok_q >= 0 ? tok_q : it.tok[0]) * a.h_out + c0 + 4 * q;
    constexpr int NL = NCB / 4;  // lines of a full unit
    uint2 yv[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) yv[i] = *reinterpret_cast<const uint2 *>(yrow + (4 * i < n_cb ? 64 * i : 0));

    float vlo[TB], vhi[TB];
    if (!fetch_v_rows<(KS > 2)>(a, it, ho, vlo, vhi)) return;
    __bf16(*vb)[LORA_MAX_RANK] = reinterpret_cast<__bf16(*)[LORA_MAX_RANK]>(vs);  // [TB][128] bf16 in this wavefront's rows
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        const bool live = it.tok[t] >= 0;
        vb[t][lane] = (__bf16)((live && lane < it.rank) ? s * vlo[t] : 0.f);
        vb[t][lane + 64] = (__bf16)((KS > 2 && live && lane + 64 < it.rank) ? s * vhi[t] : 0.f);
    }
    // only this wavefront reads what it wrote, and a wavefront's LDS operations execute in order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    gv_bf16x8 vop[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const gv_bf16x8 r = *reinterpret_cast<const gv_bf16x8 *>(&vb[m & (TB - 1)][32 * ks + 8 * g]);
        const gv_bf16x8 z = {(__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f};
        vop[ks] = m < TB ? r : z;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();  // the products are parked over the staged v
    float(*dp)[GEMV_DP_ROW] = reinterpret_cast<float(*)[GEMV_DP_ROW]>(vs);  // [TB][columns of the unit] fp32
#pragma unroll
    for (int b = 0; b < NCB; ++b) {
        gv_floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(gv_bf16x8, br[b][ks]), vop[ks], acc, 0, 0, 0);
        // acc[i]: column 16b + 4g + i (of the unit) of token m
        if (m < TB) *reinterpret_cast<gv_floatx4 *>(&dp[m][16 * b + 4 * g]) = acc;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const gv_floatx4 d = *reinterpret_cast<const gv_floatx4 *>(&dp[tq][64 * i + 4 * q]);
        const unsigned lo = yv[i].x, hi = yv[i].y;
        typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
        bf16x4 o;
        o[0] = (__bf16)(__uint_as_float(lo << 16) + d[0]);
        o[1] = (__bf16)(__uint_as_float(lo & 0xffff0000u) + d[1]);
        o[2] = (__bf16)(__uint_as_float(hi << 16) + d[2]);
        o[3] = (__bf16)(__uint_as_float(hi & 0xffff0000u) + d[3]);
        if (tok_q >= 0 && 4 * i < n_cb) {
            if (a.y32) *reinterpret_cast<gv_floatx4 *>(a.y32 + (size_t)tok_q * a.h_out + c0 + 4 * q + 64 * i) = d;
            else *reinterpret_cast<bf16x4 *>(yrow + 64 * i) = o;
        }
    }
}

// Any other rank: granule loop, v of the item's tokens staged in this wavefront's LDS rows.
template <typename E>
__device__ __forceinline__ void gemv_expand_generic(const ApplyArgs &a, const GemvItem &it, int c0, int c1, const E *Bp,
                                                    const Handover &ho, float (*vs)[GEMV_DP_ROW])
{
    const int lane = threadIdx.x & 63;
    const int rs = rank_storage(it.rank), rs8 = rs >> 3;
    const float s = a.scale * it.alpha;
    E *y = static_cast<E *>(a.y);
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        if (it.tok[t] >= 0) {  // uniform
            for (int j0 = 0; j0 < rs; j0 += 64) {
                const int jj = j0 + lane;  // v rows are at least 128 entries long
                float val;
                if (ho.vtag) {
                    const unsigned long long *const vp[1] = {ho.vtag + (size_t)it.tok[t] * a.v_stride + jj};
                    const bool need[1] = {jj < it.rank};
                    float got[1];
                    if (!fetch_v(ho, vp, need, got)) return;
                    val = got[0];
                } else {
                    val = a.v[(size_t)it.tok[t] * a.v_stride + jj];
                }
                if (jj < rs) vs[t][jj] = jj < it.rank ? s * val : 0.f;
            }
        }
    }
    // only this wavefront reads what it wrote, and a wavefront's LDS operations execute in order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    for (int n = c0 + lane; n < c1; n += 64) {
        float acc[TB];
#pragma unroll
        for (int t = 0; t < TB; ++t) acc[t] = 0.f;
#pragma unroll 4
        for (int j8 = 0; j8 < rs8; ++j8) {
            float bf[8];
            unpack_chunk(load_chunk(Bp + ((size_t)j8 * a.h_out + n) * 8), bf);
#pragma unroll
            for (int t = 0; t < TB; ++t) {
                if (it.tok[t] >= 0) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) acc[t] += vs[t][j8 * 8 + i] * bf[i];
                }
            }
        }
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            if (it.tok[t] >= 0) {
                E *yp = y + (size_t)it.tok[t] * a.h_out + n;
                if (a.y32) a.y32[(size_t)it.tok[t] * a.h_out + n] = acc[t];
                else *yp = from_float<E>(to_float(*yp) + acc[t]);
            }
        }
    }
}

// One expand unit = (item, 1024-column super-chunk `sc`), worked on by one wavefront.
template <typename E>
__device__ __forceinline__ void gemv_expand_wave(const ApplyArgs &a, const GemvItem &it, int sc, const Handover &ho,
                                                 float (*vs)[GEMV_DP_ROW])
{
    const int rs = rank_storage(it.rank);
    const int n_cols = gemv_expand_width(it.rank);
    int c0, c1;
    gemv_expand_cols(it, sc, a.h_out, c0, c1);
    if (c0 >= c1) return;
    const E *Bp = reinterpret_cast<const E *>(a.proj_base + (int64_t)it.row * a.row_bytes) + (size_t)rs * a.h_in;
    if constexpr (sizeof(E) == 2) {
        if (rs >= 32) {  // uniform over the wavefront
            const int ks = (rs + 31) >> 5, ncb = n_cols >> 4;
            if (ks == 1) gemv_expand_mfma<1, 16>(a, it, c0, c1, Bp, ho, vs);
            else if (ks == 2 && ncb == 12) gemv_expand_mfma<2, 12>(a, it, c0, c1, Bp, ho, vs);
            else if (ks == 2) gemv_expand_mfma<2, 8>(a, it, c0, c1, Bp, ho, vs);
            else if (ks == 3) gemv_expand_mfma<3, 4>(a, it, c0, c1, Bp, ho, vs);
            else gemv_expand_mfma<4, 4>(a, it, c0, c1, Bp, ho, vs);
            return;
        }
    }
    switch (rs) {  // uniform over the wavefront
        case 8: gemv_expand_body<E, 1>(a, it, c0, c1, Bp, ho); break;
        case 16: gemv_expand_body<E, 2>(a, it, c0, c1, Bp, ho); break;
        case 32: gemv_expand_body<E, 4>(a, it, c0, c1, Bp, ho); break;
        case 64: gemv_expand_body<E, 8>(a, it, c0, c1, Bp, ho); break;
        case 128: gemv_expand_body<E, 16>(a, it, c0, c1, Bp, ho); break;
        default: gemv_expand_generic<E>(a, it, c0, c1, Bp, ho, vs); break;
    }
}

// ---------------------------------------------------------------------------------------
// kernels
// ---------------------------------------------------------------------------------------
// One item per block of W wavefronts.
template <typename E>
__global__ __launch_bounds__(64 * SHRINK_MAX_W) void gemv_shrink_kernel(ApplyArgs a, const GemvItem *__restrict__ items)
{
    __shared__ float red[SHRINK_MAX_W][16];
    const GemvItem it = items[blockIdx.x];
    gemv_shrink_dispatch<E>(a, it, Handover{nullptr, 0u, nullptr}, red);
}

template <typename E>
__global__ __launch_bounds__(64) void gemv_expand_kernel(ApplyArgs a, const GemvItem *__restrict__ items)
{
    __shared__ __attribute__((aligned(16))) float vs[TB][GEMV_DP_ROW];
    const GemvItem it = items[blockIdx.x];
    gemv_expand_wave<E>(a, it, blockIdx.y, Handover{nullptr, 0u, nullptr}, vs);
}

// Fused: blocks of 4 wavefronts; blocks [0, n_gs) are the shrink blocks, one item each (long
// rows take several passes); the rest hold 4 expand wavefronts each.  Blocks are dispatched in index order, so every shrink block is running or
// done by the time an expand wavefront starts to wait, and shrink blocks wait for nothing.
template <typename E>
__global__ __launch_bounds__(256) void gemv_fused_kernel(ApplyArgs a, const GemvItem *__restrict__ gs,
                                                         const GemvItem *__restrict__ ge, int n_gs, int n_ge, int n_super,
                                                         Handover ho)
{
    __shared__ float red[4][16];
    __shared__ __attribute__((aligned(16))) float vs[4][TB][GEMV_DP_ROW];
    if ((int)blockIdx.x < n_gs) {
        const GemvItem it = gs[blockIdx.x];
        gemv_shrink_dispatch<E>(a, it, ho, red);
    } else {
        // the wavefront number and everything read through it are the same in all lanes: say so, and the
        // item's fields and the addresses built from them stay in scalar registers
        const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const int unit = ((int)blockIdx.x - n_gs) * 4 + w;
        const int item = unit / n_super;
        if (item >= n_ge) return;
        GemvItem it = ge[item];
#pragma unroll
        for (int t = 0; t < GEMV_BATCH; ++t) it.tok[t] = __builtin_amdgcn_readfirstlane(it.tok[t]);
        it.row = __builtin_amdgcn_readfirstlane(it.row);
        it.rank = __builtin_amdgcn_readfirstlane(it.rank);
        it.a = __builtin_amdgcn_readfirstlane(it.a);
        it.alpha = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, it.alpha)));
        gemv_expand_wave<E>(a, it, unit - item * n_super, ho, vs[w]);
    }
}

// wavefronts per shrink item: as many as the row has pairs of runs of 64 chunks, at most 16
static int shrink_waves(int h_in, int dtype)
{
    const int runs = (h_in / 8 + 63) / 64;
    const int u = dtype == LORA_BF16 ? shrink_u<__bf16>() : shrink_u<float>();
    return std::min(SHRINK_MAX_W, (runs + u - 1) / u);
}

hipError_t launch_gemv_shrink(int dtype, const ApplyArgs &a, const GemvItem *items, int n_items, hipStream_t st,
                              const KernelTimer *tm)
{
    if (n_items <= 0) return hipSuccess;
    const dim3 grid(n_items), block(64 * shrink_waves(a.h_in, dtype));
    if (dtype == LORA_BF16) launch_k(tm, LORA_K_GEMV_SHRINK, gemv_shrink_kernel<__bf16>, grid, block, st, a, items);
    else launch_k(tm, LORA_K_GEMV_SHRINK, gemv_shrink_kernel<float>, grid, block, st, a, items);
    return hipGetLastError();
}

hipError_t launch_gemv_expand(int dtype, const ApplyArgs &a, const GemvItem *items, int n_items, hipStream_t st,
                              const KernelTimer *tm)
{
    if (n_items <= 0) return hipSuccess;
    const dim3 grid(n_items, (a.h_out + GEMV_SUPER_COLS - 1) / GEMV_SUPER_COLS);
    if (dtype == LORA_BF16) launch_k(tm, LORA_K_GEMV_EXPAND, gemv_expand_kernel<__bf16>, grid, dim3(64), st, a, items);
    else launch_k(tm, LORA_K_GEMV_EXPAND, gemv_expand_kernel<float>, grid, dim3(64), st, a, items);
    return hipGetLastError();
}

hipError_t launch_gemv_fused(int dtype, const ApplyArgs &a, const GemvItem *gs, int n_gs, const GemvItem *ge, int n_ge,
                             unsigned long long *vtag, uint32_t epoch, int32_t *fault, hipStream_t st, const KernelTimer *tm)
{
    if (n_gs <= 0 || n_ge <= 0) return hipSuccess;
    const int n_super = (a.h_out + GEMV_SUPER_COLS - 1) / GEMV_SUPER_COLS;
    const int n_expand_blocks = (n_ge * n_super + 3) / 4;
    const dim3 grid(n_gs + n_expand_blocks), block(256);
    const Handover ho{vtag, epoch, fault};
    if (dtype == LORA_BF16)
        launch_k(tm, LORA_K_GEMV_FUSED, gemv_fused_kernel<__bf16>, grid, block, st, a, gs, ge, n_gs, n_ge, n_super, ho);
    else
        launch_k(tm, LORA_K_GEMV_FUSED, gemv_fused_kernel<float>, grid, block, st, a, gs, ge, n_gs, n_ge, n_super, ho);
    return hipGetLastError();
}

}  // namespace lora
