// Base projection and adapter update in one matrix-core kernel for gfx950 (bf16 in, fp32 accumulate):
//     y[t] = x[t] . W  +  s_i . v[t] . B_i          v[t] = x[t] . A_i from the shrink kernels
// for row tiles of up to 64 tokens that share one adapter (or have none).  The adapter product enters
// as one more slab of the contraction after the k loop over h_in, so the output is written once and
// never read: the separate addition of the adapter result to the base output (paper section 3.1)
// disappears.  This is the variant of the hot path whose roof is the matrix cores, not HBM.
//
// Block = 8 wavefronts on 256 rows (four row tiles) x 256 output columns; wavefront w owns the row
// half w%2 and the column quarter w/2: 8 x 4 products of 16 x 16 (v_mfma_f32_16x16x32_bf16, 128
// accumulator registers).  The 32x32x16 form of the product has the higher peak rate, but beside the
// stage loads it is the slower one: the k loop of this kernel as a microbenchmark takes 197 us with it
// and 173 us with the 16x16x32 form on the prefill shape (loads alone 120 us, products alone 120 us).
// Two wavefronts per SIMD: with one, every wait -- the barrier of a stage, the first operand reads
// after it -- idles the matrix core.  x rows (gathered by token) and Wt rows (Wt[n][k] = W[k][n], the
// layout a linear layer keeps its weight in) are both contiguous along k: every stage brings 64 k of
// both into LDS, double-buffered, one barrier per stage, by global_load_lds_dwordx4 -- the load writes
// LDS itself (at the wavefront's base + 16 bytes x lane; checked on the part), so no registers stage
// the data (loads that return into registers while products run took more than twice as long).
// LDS rows are 128 bytes without padding; bank conflicts are avoided by a swizzle instead: 16-byte
// slot s of row r holds piece s ^ ((r/2) % 8) of the row's 64 k, so the 16 rows an operand read
// touches at once fall into 16 different bank groups.  Per 32-wide k step a wavefront reads 8 + 4
// operands from LDS for 32 products.
// Operand layout of the instruction: A (16 x 32): lane l holds row l%16, k = 8*(l/16) .. +7;
// B (32 x 16): lane l holds column l%16, same k; D: lane l holds column l%16, rows 4*(l/16) .. +3.
// The products are formed transposed -- the W block is the row operand, the x block the column
// operand -- so that a lane's four accumulator registers are four consecutive output columns of one
// token: 8 bytes of bf16, parked in LDS and stored from there in whole 128-byte lines.
// After the k loop the scaled intermediate s.v of the block's rows is staged in LDS as bf16 and every
// wavefront adds, per row tile, the products with that tile's Bp, whose rank-packed layout gives the
// row operand directly from global memory (a lane's 8 ranks are 16 contiguous bytes).
// Tokens on the GEMV path sit in row tiles without an adapter; their adapter term is computed by the
// GEMV kernels beforehand into the (zeroed) output rows, and this kernel adds it to the accumulators of
// those rows before the one rounding of the stored value (row tiles marked a = 1).
//
// One block fills a CU (its two stages take 144 KB of LDS), so a grid of N tiles runs in ceil(N / CUs)
// rounds and the last round may be nearly empty (368 tiles on 256 CUs: a second round of 112).  The tiles of
// that last round are therefore split along k into S = 2 or 4 parts, one block each, as many as fit one round:
// the last part of a tile is its owner -- it is dispatched last, so the other parts are running or done
// when it waits for them, and they wait for nothing -- and adds the other parts' fp32 accumulators, which
// travel through a scratch area as device-scope atomic stores and loads (past the per-XCD L2s) behind a
// flag per part that the owner resets; its wait is bounded and raises the cache's fault flag.
#include <algorithm>

#include "lora_device.h"

namespace lora {

namespace {
constexpr int LBM = 256, LBN = 256, LBK = 64;
constexpr int LROW = LBK * 2;                   // bytes per row of a stage in LDS (swizzled, not padded)
constexpr int L_A = LBM * LROW;                 // x part of a stage
constexpr int L_STAGE = (LBM + LBN) * LROW;     // 73728 bytes
constexpr int SV_ROW = LORA_MAX_RANK * 2 + 16;  // bytes per row of the staged s.v
static_assert(8 * 128 * 128 <= 2 * L_STAGE && LBM * SV_ROW <= 2 * L_STAGE, "s.v is staged in the stage buffers");
}  // namespace


// split of the last round: blocks [0, n_whole) work on whole tiles; block n_whole + S * j + p on part p of tile n_whole + j
struct LinearSplit {
    int n_whole, parts;          // parts = 1: no split
    unsigned long long *partial;  // [tile j][part p < parts - 1][accumulator 32][half 2][thread 512] 8-byte words
    uint32_t *flags;              // [tile j][part p < parts - 1], zero between launches
    int32_t *fault;
};

__global__ __launch_bounds__(512) void linear_tiles_kernel(ApplyArgs a, const __bf16 *__restrict__ Wt,
                                                           const DevItem *__restrict__ tiles, int n_rt, int n_mt, LinearSplit sp)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];  // two stages
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 15, g = lane >> 4;
    const int rh = w & 1, cq = w >> 1;
    int tile_no = (int)blockIdx.x, part = 0, tail = -1;
    if (tile_no >= sp.n_whole) {
        tail = (tile_no - sp.n_whole) / sp.parts;
        part = (tile_no - sp.n_whole) - tail * sp.parts;
        tile_no = sp.n_whole + tail;
    }
    const bool owner = part == sp.parts - 1 || tail < 0;
    const int bm = tile_no % n_mt, bn = tile_no / n_mt;
    const int n0 = bn * LBN;

    // the four row tiles of the block (a missing one counts as empty), and the two of this wavefront's
    // row half once more under fixed names (indexing the four by the wavefront number would put them
    // in scratch memory)
    auto get_tile = [&](int idx) {
        DevItem t = tiles[min(idx, n_rt - 1)];
        if (idx >= n_rt) {
            t.n_tok = 0;
            t.rank = 0;
        }
        return t;
    };
    const DevItem it0 = get_tile(4 * bm), it1 = get_tile(4 * bm + 1), it2 = get_tile(4 * bm + 2), it3 = get_tile(4 * bm + 3);
    const DevItem mine0 = get_tile(4 * bm + 2 * rh), mine1 = get_tile(4 * bm + 2 * rh + 1);
    auto tile_of = [&](int j) -> const DevItem & { return j == 0 ? it0 : j == 1 ? it1 : j == 2 ? it2 : it3; };  // j: compile-time
    const DevItem tile_of_wave = get_tile(4 * bm + (w >> 1));  // the row tile this wavefront loads half of
    const int dead_tok = it0.tok0;  // rows past a tile's end read a live token's x; they are never stored

    const __bf16 *x = static_cast<const __bf16 *>(a.x);
    __bf16 *y = static_cast<__bf16 *>(a.y);
    const int n_k = a.h_in / LBK;
    // this block's stages of the k walk
    const int k_lo = tail < 0 ? 0 : n_k * part / sp.parts, k_hi = tail < 0 ? n_k : n_k * (part + 1) / sp.parts;

    // loader: wavefront w brings rows 32w + 8q + lane/8, q = 0..3, of both x and Wt: instruction q writes
    // 8 rows x 128 bytes at the wavefront-uniform LDS address of its first row, lane l to slot l%8 of
    // row l/8, for which it fetches piece (l%8) ^ ((row/2) % 8) of the row
    const int lr = lane >> 3, ls = lane & 7;
    const int piece_even = ls ^ ((lane >> 4) & 7), piece_odd = ls ^ (((lane >> 4) + 4) & 7);  // (row/2)%8 for q even / odd
    const __bf16 *xg[4];
    {
        int ti[4], tok[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) ti[q] = 32 * (w & 1) + 8 * q + lr;
        tile_tokens_of(a.tok_list, tile_of_wave, ti, dead_tok, tok);  // (rows past the tile's end repeat its last)
#pragma unroll
        for (int q = 0; q < 4; ++q) xg[q] = x + (size_t)tok[q] * a.h_in + ((q & 1) ? piece_odd : piece_even) * 8;
    }
    // Wt rows n0 + 32w + 8q + lr; h_out is a multiple of 64, so a run of 32 rows is inside or outside as a whole
    const int w_row0 = min(n0 + 32 * w, a.h_out - 32);
    const __bf16 *wg_even = Wt + (size_t)(w_row0 + lr) * a.h_in + piece_even * 8;
    const __bf16 *wg_odd = Wt + (size_t)(w_row0 + lr) * a.h_in + piece_odd * 8;
    // (All blocks walk k in step: the blocks of a row or column of the grid then find each other's
    // panel slices in L2.  Starting every block at another stage, as the tile shrink does, was no faster.)
    auto load_stage = [&](int kt, int buf) {
        const int k = kt * LBK;
        unsigned char *sa = lds + buf * L_STAGE + (32 * w) * LROW;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            __builtin_amdgcn_global_load_lds(xg[q] + k, (__attribute__((address_space(3))) void *)(sa + q * 8 * LROW), 16, 0, 0);
#pragma unroll
        for (int q = 0; q < 4; ++q)
            __builtin_amdgcn_global_load_lds(((q & 1) ? wg_odd : wg_even) + (size_t)(8 * q) * a.h_in + k,
                                             (__attribute__((address_space(3))) void *)(sa + L_A + q * 8 * LROW), 16, 0, 0);
    };

    floatx4 acc[8][4];  // [block of 16 rows][block of 16 columns]
#pragma unroll
    for (int mb = 0; mb < 8; ++mb)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[mb][nb][e] = 0.f;

    load_stage(k_lo, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    // operand reads: row R, k piece 4ks + g sits in slot (4ks + g) ^ ((R/2) % 8); R/2 % 8 = m/2 for all of a lane's rows
    const int swz = (m >> 1) & 7;
    for (int kt = k_lo; kt < k_hi; ++kt) {
        // the next stage is requested before this one is multiplied, into the buffer that was read
        // in the previous iteration (past the end: the last stage again, unconditionally)
        const int buf = (kt - k_lo) & 1;
        load_stage(min(kt + 1, k_hi - 1), buf ^ 1);
        const unsigned char *sa = lds + buf * L_STAGE + (128 * rh + m) * LROW;
        const unsigned char *sb = lds + buf * L_STAGE + L_A + (64 * cq + m) * LROW;
        // (The compiler's own order -- operand reads in twos and fours between groups of eight products -- is
        // as fast as reading the operands of every group one group ahead by hand.)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 xo[8], wo[4];
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) wo[nb] = *reinterpret_cast<const bf16x8 *>(sb + nb * 16 * LROW + (((4 * ks + g) ^ swz) << 4));
#pragma unroll
            for (int mb = 0; mb < 8; ++mb) xo[mb] = *reinterpret_cast<const bf16x8 *>(sa + mb * 16 * LROW + (((4 * ks + g) ^ swz) << 4));
#pragma unroll
            for (int mb = 0; mb < 8; ++mb)
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) acc[mb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wo[nb], xo[mb], acc[mb][nb], 0, 0, 0);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wavefront's part of the next stage has landed
        __syncthreads();
    }

    // ---- a tile split along k: the parts hand their accumulators to the owner
    if (tail >= 0) {
        typedef float floatx2 __attribute__((ext_vector_type(2)));
        const size_t per_part = (size_t)32 * 2 * 512;  // words
        if (!owner) {
            unsigned long long *dst = sp.partial + ((size_t)tail * (sp.parts - 1) + part) * per_part + tid;
#pragma unroll
            for (int mb = 0; mb < 8; ++mb)
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) {
                    const floatx4 c = acc[mb][nb];
                    const floatx2 lo = {c[0], c[1]}, hi = {c[2], c[3]};
                    __hip_atomic_store(dst + ((mb * 4 + nb) * 2 + 0) * 512, __builtin_bit_cast(unsigned long long, lo), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(dst + ((mb * 4 + nb) * 2 + 1) * 512, __builtin_bit_cast(unsigned long long, hi), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the stores above have been performed where every XCD sees them
            __syncthreads();
            if (tid == 0) __hip_atomic_store(sp.flags + tail * (sp.parts - 1) + part, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        __shared__ int got_all;
        if (tid == 0) {
            int ok = 1;
            for (int p = 0; p < sp.parts - 1 && ok; ++p) {
                ok = 0;
                for (int spin = 0; spin < (1 << 20); ++spin) {
                    if (__hip_atomic_load(sp.flags + tail * (sp.parts - 1) + p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
                        ok = 1;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(8);
                }
            }
            if (!ok) __hip_atomic_store(sp.fault, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);  // pinned host memory
            got_all = ok;
        }
        __syncthreads();
        if (got_all) {
            for (int p = 0; p < sp.parts - 1; ++p) {
                const unsigned long long *src = sp.partial + ((size_t)tail * (sp.parts - 1) + p) * per_part + tid;
#pragma unroll
                for (int mb = 0; mb < 8; ++mb)
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb) {
                        const floatx2 lo = __builtin_bit_cast(floatx2, __hip_atomic_load(src + ((mb * 4 + nb) * 2 + 0) * 512, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                        const floatx2 hi = __builtin_bit_cast(floatx2, __hip_atomic_load(src + ((mb * 4 + nb) * 2 + 1) * 512, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                        acc[mb][nb][0] += lo[0];
                        acc[mb][nb][1] += lo[1];
                        acc[mb][nb][2] += hi[0];
                        acc[mb][nb][3] += hi[1];
                    }
            }
        }
        __syncthreads();
        if (tid < sp.parts - 1) __hip_atomic_store(sp.flags + tail * (sp.parts - 1) + tid, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    // ---- the adapter slab.  Bp operands of a row tile: granule 4ks + g (the 8 ranks a lane's operand holds,
    // contiguous per column; past the stored rank the last granule, which meets zeros of s.v), all four k
    // steps requested at once -- and for the wavefront's first tile before s.v is staged, so that the
    // requests fly while the staging waits for its own loads.
    auto bp_of = [&](const DevItem &t) {
        return reinterpret_cast<const __bf16 *>(a.proj_base + (int64_t)t.row * a.row_bytes) + (size_t)rank_storage(t.rank) * a.h_in;
    };
    auto load_bp = [&](const DevItem &t, bf16x8(&bo)[4][4]) {
        const int rs8 = rank_storage(max(t.rank, 1)) >> 3;
        const __bf16 *Bp = bp_of(t);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                const int col = min(n0 + 64 * cq + 16 * nb + m, a.h_out - 1);
                bo[ks][nb] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(Bp + ((size_t)min(4 * ks + g, rs8 - 1) * a.h_out + col) * 8));
            }
    };
    const bool live0 = mine0.rank != 0 && mine0.n_tok != 0, live1 = mine1.rank != 0 && mine1.n_tok != 0;  // wavefront-uniform
    bf16x8 bo[4][4];
    if (live0) load_bp(mine0, bo);
    // s.v of the block's rows to LDS as bf16 (zero past a tile's rank or end)
    unsigned char *sv = lds;
    {
        // chunk tid%16 (8 ranks) of rows tid/16 and tid/16 + 32 of each row tile that has an adapter: per tile the
        // two token ids in one round, then both rows' pieces in one round (unconditional, from addresses inside v)
        const int c8 = tid & 15, r0 = tid >> 4;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const DevItem &t = tile_of(jj);
            if (t.rank == 0 || t.n_tok == 0) continue;  // uniform over the block; nothing of such a tile is read below
            const int ks32 = (t.rank + 31) >> 5;        // k steps this tile's products will read
            const int ti[2] = {r0, r0 + 32};
            int tok[2];
            tile_tokens_of(a.tok_list, t, ti, dead_tok, tok);
            uint4 pc[2];  // s.v comes as bf16 from the shrink or the reduce (rows of the fp32 pitch)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                pc[h] = *reinterpret_cast<const uint4 *>(reinterpret_cast<const __bf16 *>(a.v) + (size_t)tok[h] * (2 * a.v_stride) + c8 * 8);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (c8 < 4 * ks32) {
                    const bf16x8 f = __builtin_bit_cast(bf16x8, pc[h]);
                    bf16x8 o;
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] = (ti[h] < t.n_tok && c8 * 8 + e < t.rank) ? f[e] : (__bf16)0.f;
                    *reinterpret_cast<bf16x8 *>(sv + (64 * jj + ti[h]) * SV_ROW + c8 * 16) = o;
                }
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int tl = 0; tl < 2; ++tl) {
        const DevItem &t = tl ? mine1 : mine0;
        if (!(tl ? live1 : live0)) continue;
        if (tl == 1) load_bp(mine1, bo);
        const int ks32 = (t.rank + 31) >> 5;
        const unsigned char *svr = sv + (128 * rh + 64 * tl + m) * SV_ROW + g * 16;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks < ks32) {
#pragma unroll
                for (int mbl = 0; mbl < 4; ++mbl) {
                    const bf16x8 xo = *reinterpret_cast<const bf16x8 *>(svr + mbl * 16 * SV_ROW + ks * 64);
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb)
                        acc[4 * tl + mbl][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bo[ks][nb], xo, acc[4 * tl + mbl][nb], 0, 0, 0);
                }
            }
        }
    }

    // ---- store.  The products are formed transposed (the W block is the instruction's row operand, the x
    // block its column operand): lane (m, g) holds, in the four registers of block (mb, nb), row 16*mb + m of the
    // wavefront's 128 and the four consecutive columns 16*nb + 4g .. of its 64 -- 8 bytes of bf16.  The
    // wavefront parks its 128 x 64 outputs in LDS and stores whole 128-byte row pieces, 8 rows per
    // instruction (stored from the registers, an instruction would write 32 bytes to each of 16 rows).
    // Park layout, free of bank conflicts both ways: row r is 128 bytes, its 8-byte cell c sits at
    // c ^ (2 * ((r/2) % 8)), i.e. its 16-byte slot s at s ^ ((r/2) % 8).  Row tiles whose rows already hold
    // the adapter term (GEMV tokens) are few and go straight from the registers, the sum formed in fp32
    // before the one rounding.
    __syncthreads();  // every wavefront is done with the staged s.v
    unsigned char *park = lds + w * (128 * 128);
    const bool cols_live = n0 + 64 * cq < a.h_out;  // h_out is a multiple of 64
    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int tl = 0; tl < 2; ++tl) {
        const DevItem &t = tl ? mine1 : mine0;
        if (t.n_tok == 0 || !cols_live) continue;  // wavefront-uniform
        const bool add_y = t.rank == 0 && t.a == 1;
        if (add_y) {
            // rows whose adapter term is already in y (or, as fp32, at the same place of the workspace): the four
            // token ids in one round, then per row block the four old values in one round and the four stores
            int ti4[4], tok4[4];
#pragma unroll
            for (int mbl = 0; mbl < 4; ++mbl) ti4[mbl] = 16 * mbl + m;
            tile_tokens_of(a.tok_list, t, ti4, dead_tok, tok4);
#pragma unroll
            for (int mbl = 0; mbl < 4; ++mbl) {
                if (ti4[mbl] >= t.n_tok) continue;
                __bf16 *yr = y + (size_t)tok4[mbl] * a.h_out + n0 + 64 * cq + 4 * g;
                floatx4 term[4];
                if (a.y32) {
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb) term[nb] = *reinterpret_cast<const floatx4 *>(a.y32 + (yr - y) + 16 * nb);
                } else {
                    bf16x4 old[4];
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb) old[nb] = *reinterpret_cast<const bf16x4 *>(yr + 16 * nb);
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                        for (int e = 0; e < 4; ++e) term[nb][e] = (float)old[nb][e];
                }
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) {
                    const floatx4 c = acc[4 * tl + mbl][nb];
                    bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = (__bf16)(c[e] + term[nb][e]);
                    *reinterpret_cast<bf16x4 *>(yr + 16 * nb) = o;
                }
            }
            continue;
        }
#pragma unroll
        for (int mbl = 0; mbl < 4; ++mbl) {
            const int ti = 16 * mbl + m, row = 64 * tl + ti;
            unsigned char *pr = park + row * 128;
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                const floatx4 c = acc[4 * tl + mbl][nb];
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (__bf16)c[e];
                *reinterpret_cast<bf16x4 *>(pr + (((4 * nb + g) ^ (((row >> 1) & 7) << 1)) << 3)) = o;
            }
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // only this wavefront reads what it wrote; its LDS operations execute in order
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int tl = 0; tl < 2; ++tl) {
        const DevItem &t = tl ? mine1 : mine0;
        if (t.n_tok == 0 || !cols_live || (t.rank == 0 && t.a == 1)) continue;  // wavefront-uniform
        const int rl = lane >> 3, sl = lane & 7;
        int ti8[8], tok8[8];  // the rows' token ids all before the first store (a lookup between two stores makes the second wait for the first)
#pragma unroll
        for (int i = 0; i < 8; ++i) ti8[i] = 8 * i + rl;
        tile_tokens_of(a.tok_list, t, ti8, dead_tok, tok8);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = 64 * tl + ti8[i];
            if (ti8[i] < t.n_tok) {
                const uint4 v = *reinterpret_cast<const uint4 *>(park + row * 128 + ((sl ^ ((row >> 1) & 7)) << 4));
                // (a streaming store: the rows leave the caches as they are written instead of lying there dirty
                // until the next kernel's loads push them out -- the tile shrink that follows runs 2 to 3 us shorter)
                typedef unsigned u32x4_nt __attribute__((ext_vector_type(4)));
                const u32x4_nt vn = {v.x, v.y, v.z, v.w};
                __builtin_nontemporal_store(vn, reinterpret_cast<u32x4_nt *>(y + (size_t)tok8[i] * a.h_out + n0 + 64 * cq + 8 * sl));
            }
        }
    }
}

// y[token][0 .. h_out) = 0 for the listed tokens (the rows the GEMV expand then adds its term to)
__global__ __launch_bounds__(256) void zero_rows_kernel(__bf16 *__restrict__ y, const int32_t *__restrict__ toks, int n, int h_out)
{
    const int per_row = h_out / 8;  // 16-byte pieces
    for (int i = blockIdx.x * 256 + threadIdx.x; i < n * per_row; i += gridDim.x * 256) {
        const int r = i / per_row, c = i - r * per_row;
        *reinterpret_cast<uint4 *>(y + (size_t)toks[r] * h_out + c * 8) = make_uint4(0, 0, 0, 0);
    }
}

hipError_t launch_zero_rows(void *y, const int32_t *toks, int n, int h_out, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    const int blocks = std::min(1024, (n * (h_out / 8) + 255) / 256);
    hipLaunchKernelGGL(zero_rows_kernel, dim3(blocks), dim3(256), 0, st, static_cast<__bf16 *>(y), toks, n, h_out);
    return hipGetLastError();
}

// parts the tiles of the last round are split into (1: none), and how many tiles that round has
static void linear_split_shape(int n_tiles, int n_k, int n_cu, int &parts, int &n_tail)
{
    n_tail = n_tiles % n_cu;
    parts = 1;
    if (n_tail == 0) return;
    const int fit = n_cu / n_tail;  // blocks per tile that still fit one round
    if (fit >= 4 && n_k % 4 == 0) parts = 4;
    else if (fit >= 2 && n_k % 2 == 0) parts = 2;
    if (parts == 1) n_tail = 0;
}

size_t linear_split_bytes(int n_rt, int h_in, int h_out, int n_cu)
{
    int parts, n_tail;
    linear_split_shape(((n_rt + 3) / 4) * ((h_out + LBN - 1) / LBN), h_in / LBK, n_cu, parts, n_tail);
    return (size_t)n_tail * (parts - 1) * 32 * 2 * 512 * sizeof(unsigned long long);
}

hipError_t launch_linear_tiles(const ApplyArgs &a, const void *Wt, const DevItem *row_tiles, int n_rt, void *split_scratch,
                               size_t split_scratch_bytes, uint32_t *split_flags, int n_split_flags, int32_t *fault, int n_cu,
                               hipStream_t st, const KernelTimer *tm)
{
    if (n_rt <= 0) return hipSuccess;
    static bool attr_set = false;
    if (!attr_set) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(linear_tiles_kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 2 * L_STAGE);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int n_mt = (n_rt + 3) / 4, n_nt = (a.h_out + LBN - 1) / LBN, n_tiles = n_mt * n_nt;
    int parts, n_tail;
    linear_split_shape(n_tiles, a.h_in / LBK, n_cu, parts, n_tail);
    if (parts > 1 && (linear_split_bytes(n_rt, a.h_in, a.h_out, n_cu) > split_scratch_bytes || n_tail * (parts - 1) > n_split_flags || !split_scratch))
        parts = 1, n_tail = 0;  // no room for the partial sums: whole tiles only
    const LinearSplit sp{n_tiles - n_tail, parts, static_cast<unsigned long long *>(split_scratch), split_flags, fault};
    const int blocks = n_tiles - n_tail + n_tail * parts;
    hipEvent_t s = nullptr, e = nullptr;
    if (tm) tm->pair(tm->ctx, LORA_K_LINEAR, &s, &e);
    if (s && e)
        hipExtLaunchKernelGGL(linear_tiles_kernel, dim3(blocks), dim3(512), 2 * L_STAGE, st, s, e, 0, a,
                              static_cast<const __bf16 *>(Wt), row_tiles, n_rt, n_mt, sp);
    else
        hipLaunchKernelGGL(linear_tiles_kernel, dim3(blocks), dim3(512), 2 * L_STAGE, st, a, static_cast<const __bf16 *>(Wt),
                           row_tiles, n_rt, n_mt, sp);
    return hipGetLastError();
}

}  // namespace lora
