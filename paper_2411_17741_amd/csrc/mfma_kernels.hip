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
#include "lora_device.h"

namespace lora {

namespace {
constexpr int VS_ROW = LORA_MAX_RANK * 2 + 16;  // bytes per token row of the staged V tile (padded)
constexpr int EXPAND_COLS = 512;                // expand: columns per block, in passes of 128
}  // namespace

// ---------------------------------------------------------------------------------------
// shrink.  Block = 4 wavefronts on one tile and one k range; the range is cut in four and
// every wavefront works alone on its quarter: all (up to 4) token blocks x all (up to NBMAX)
// rank blocks, both operands loaded straight from global memory into MFMA registers -- x from
// HBM, At from L2 -- with the next step's loads in flight while the current step multiplies.
// No LDS and no barrier in the loop.  Per step a lane group g covers k = k0 + (KS/4)*g .. and
// MFMA i of the step uses the i-th 8 of them.  The four partial results are summed through
// LDS at the end.  NBMAX (1, 2, 4, 8 rank blocks of 16) is a template parameter so that small
// ranks do not pay for the accumulators of large ones; a block leaves at once if its tile
// belongs to another class.
// ---------------------------------------------------------------------------------------
template <int NBMAX, int KS>
__global__ __launch_bounds__(256) void mfma_shrink_kernel(ApplyArgs a, const DevItem *__restrict__ tiles, int k_len,
                                                          int use_atomic)
{
    constexpr int NI = KS / 32;   // MFMA k steps per loop step
    constexpr int LB = KS / 4;    // elements per lane per operand row per step
    __shared__ __attribute__((aligned(16))) float red[2][4 * NBMAX * 4][64];

    const DevItem it = tiles[blockIdx.x];
    const int NB = (it.rank + 15) >> 4;
    if (NB > NBMAX || (NBMAX > 1 && NB <= NBMAX / 2)) return;  // another class (uniform)

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int rs = rank_storage(it.rank);
    const int n_mb = (it.n_tok + 15) >> 4;
    const int kq = k_len >> 2;  // k_len is a multiple of 4*KS
    const int k_lo = blockIdx.y * k_len + w * kq;
    const int k_hi = min(a.h_in, k_lo + kq);
    const int n_steps = k_hi > k_lo ? (k_hi - k_lo + KS - 1) / KS : 0;

    const __bf16 *At = reinterpret_cast<const __bf16 *>(a.proj_base + (int64_t)it.row * a.row_bytes);
    const __bf16 *x = static_cast<const __bf16 *>(a.x);

    const __bf16 *xp[4];
    bool x_ok[4];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
        const int ti = 16 * mb + m;
        x_ok[mb] = ti < it.n_tok;
        const int tok = x_ok[mb] ? (ti == 0 ? it.tok0 : a.tok_list[it.tok_off + ti]) : 0;
        xp[mb] = x + (size_t)tok * a.h_in + LB * g;
    }
    const __bf16 *ap[NBMAX];
    bool a_ok[NBMAX];
#pragma unroll
    for (int nb = 0; nb < NBMAX; ++nb) {
        const int row = 16 * nb + m;
        a_ok[nb] = row < rs;
        ap[nb] = At + (size_t)(a_ok[nb] ? row : 0) * a.h_in + LB * g;
    }

    floatx4 acc[4][NBMAX];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBMAX; ++nb) acc[mb][nb] = floatx4{0.f, 0.f, 0.f, 0.f};

    uint4 xr[2][4][NI], ar[2][NBMAX][NI];
    auto load_step = [&](int k, uint4(&xd)[4][NI], uint4(&ad)[NBMAX][NI]) {
        // a step may stick out of the range by 64 elements when KS = 128: pieces are predicated
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int i = 0; i < NI; ++i)
                xd[mb][i] = (x_ok[mb] && mb < n_mb && k + LB * g + 8 * i < k_hi)
                                ? *reinterpret_cast<const uint4 *>(xp[mb] + k + 8 * i)
                                : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int nb = 0; nb < NBMAX; ++nb)
#pragma unroll
            for (int i = 0; i < NI; ++i)
                ad[nb][i] = (a_ok[nb] && nb < NB && k + LB * g + 8 * i < k_hi)
                                ? *reinterpret_cast<const uint4 *>(ap[nb] + k + 8 * i)
                                : make_uint4(0, 0, 0, 0);
    };
    auto mul_step = [&](uint4(&xd)[4][NI], uint4(&ad)[NBMAX][NI]) {
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int mb = 0; mb < 4; ++mb) {
                if (mb < n_mb) {
                    const bf16x8 av = __builtin_bit_cast(bf16x8, xd[mb][i]);
#pragma unroll
                    for (int nb = 0; nb < NBMAX; ++nb)
                        if (nb < NB)
                            acc[mb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                av, __builtin_bit_cast(bf16x8, ad[nb][i]), acc[mb][nb], 0, 0, 0);
                }
            }
    };

    if (n_steps > 0) load_step(k_lo, xr[0], ar[0]);
    for (int sidx = 0; sidx < n_steps; sidx += 2) {
        if (sidx + 1 < n_steps) load_step(k_lo + (sidx + 1) * KS, xr[1], ar[1]);
        mul_step(xr[0], ar[0]);
        if (sidx + 2 < n_steps) load_step(k_lo + (sidx + 2) * KS, xr[0], ar[0]);
        if (sidx + 1 < n_steps) mul_step(xr[1], ar[1]);
    }

    // sum the four wavefronts' partials: 2,3 -> LDS -> 0,1 add; 1 -> LDS -> 0 adds and writes
    auto spill = [&](int slot) {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int nb = 0; nb < NBMAX; ++nb)
#pragma unroll
                for (int r = 0; r < 4; ++r) red[slot][(mb * NBMAX + nb) * 4 + r][lane] = acc[mb][nb][r];
    };
    auto absorb = [&](int slot) {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int nb = 0; nb < NBMAX; ++nb)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[mb][nb][r] += red[slot][(mb * NBMAX + nb) * 4 + r][lane];
    };
    if (w >= 2) spill(w - 2);
    __syncthreads();
    if (w < 2) absorb(w);
    __syncthreads();
    if (w == 1) spill(0);
    __syncthreads();
    if (w != 0) return;
    absorb(0);

#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int ti = 16 * mb + 4 * g + r;
            if (ti < it.n_tok) {
                float *vr = a.v + (size_t)(ti == 0 ? it.tok0 : a.tok_list[it.tok_off + ti]) * a.v_stride;
#pragma unroll
                for (int nb = 0; nb < NBMAX; ++nb) {
                    const int jr = 16 * nb + m;
                    if (nb < NB && jr < it.rank) {
                        if (use_atomic) unsafeAtomicAdd(vr + jr, acc[mb][nb][r]);
                        else vr[jr] = acc[mb][nb][r];
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// expand.  Block = 4 wavefronts, tile of up to 64 tokens x EXPAND_COLS columns in passes of
// 128 columns; wavefront w owns token half w&1 and column half w>>1 of a pass (32 tokens x 64
// columns).  The scaled V tile is staged once in LDS as bf16.  The product is formed
// transposed (rows = output columns, columns = tokens) so that a lane ends up with runs of 8
// consecutive output columns of one token: block b of the 4 column blocks maps MFMA row
// 4q+r to column 8q + 4(b&1) + r + 32(b>>1), which makes the read-modify-write of base_out a
// pair of 16-byte accesses per lane and token, 64 contiguous bytes per row across a lane group.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void mfma_expand_kernel(ApplyArgs a, const DevItem *__restrict__ tiles)
{
    __shared__ __attribute__((aligned(16))) unsigned char vs[LORA_TILE_TOKENS * VS_ROW];

    const DevItem it = tiles[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int th = w & 1, ch = w >> 1;
    const int rs = rank_storage(it.rank), rs8 = rs >> 3;
    const int KS = (it.rank + 31) >> 5;  // MFMA k steps of 32 ranks
    const int c8 = KS * 4;               // staged chunks (8 ranks) per token
    const float s = a.scale * it.alpha;
    const __bf16 *Bp = reinterpret_cast<const __bf16 *>(a.proj_base + (int64_t)it.row * a.row_bytes) + (size_t)rs * a.h_in;
    __bf16 *y = static_cast<__bf16 *>(a.y);

    // stage s.V as bf16: vs[token][rank]
    for (int idx = tid; idx < LORA_TILE_TOKENS * c8; idx += 256) {
        const int ti = idx / c8, j8 = idx - ti * c8;
        bf16x8 o;
        if (ti < it.n_tok) {
            const float4 *vr = reinterpret_cast<const float4 *>(
                a.v + (size_t)(ti == 0 ? it.tok0 : a.tok_list[it.tok_off + ti]) * a.v_stride + j8 * 8);
            const float4 lo = vr[0], hi = vr[1];
            const float f[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (__bf16)((j8 * 8 + e < it.rank) ? s * f[e] : 0.f);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (__bf16)0.f;
        }
        *reinterpret_cast<bf16x8 *>(&vs[ti * VS_ROW + j8 * 16]) = o;
    }
    __syncthreads();

    if (32 * th >= it.n_tok) return;  // this token half is empty (no barrier follows)

    // token rows this lane reads/writes in the epilogue: 32*th + 16*tb + m
    size_t yoff[2];
    bool yok[2];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        const int ti = 32 * th + 16 * tb + m;
        yok[tb] = ti < it.n_tok;
        yoff[tb] = yok[tb] ? (size_t)(ti == 0 ? it.tok0 : a.tok_list[it.tok_off + ti]) * a.h_out : 0;
    }
    const bool tb1_live = 32 * th + 16 < it.n_tok;

    for (int cp = 0; cp < EXPAND_COLS / 128; ++cp) {
        const int nw0 = blockIdx.y * EXPAND_COLS + cp * 128 + 64 * ch;
        if (nw0 >= a.h_out) break;

        uint4 yr[2][2];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                yr[tb][h] = yok[tb] ? *reinterpret_cast<const uint4 *>(y + yoff[tb] + nw0 + 8 * g + 32 * h)
                                    : make_uint4(0, 0, 0, 0);

        floatx4 acc[4][2];
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) acc[b][tb] = floatx4{0.f, 0.f, 0.f, 0.f};

        for (int ks = 0; ks < KS; ++ks) {
            const int j8 = 4 * ks + g;
            bf16x8 aop[4], bop[2];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int n = nw0 + 8 * (m >> 2) + 4 * (b & 1) + (m & 3) + 32 * (b >> 1);
                uint4 raw = make_uint4(0, 0, 0, 0);
                if (j8 < rs8) raw = *reinterpret_cast<const uint4 *>(Bp + ((size_t)j8 * a.h_out + n) * 8);
                aop[b] = __builtin_bit_cast(bf16x8, raw);
            }
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
                bop[tb] = *reinterpret_cast<const bf16x8 *>(&vs[(32 * th + 16 * tb + m) * VS_ROW + j8 * 16]);
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                acc[b][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop[b], bop[0], acc[b][0], 0, 0, 0);
                if (tb1_live) acc[b][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop[b], bop[1], acc[b][1], 0, 0, 0);
            }
        }

#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            if (yok[tb]) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    float f[8];
                    Chunk<__bf16> c;
                    c.v = yr[tb][h];
                    unpack_chunk(c, f);
                    bf16x8 o;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        o[r] = (__bf16)(f[r] + acc[2 * h][tb][r]);
                        o[4 + r] = (__bf16)(f[4 + r] + acc[2 * h + 1][tb][r]);
                    }
                    *reinterpret_cast<bf16x8 *>(y + yoff[tb] + nw0 + 8 * g + 32 * h) = o;
                }
            }
        }
    }
}

__global__ __launch_bounds__(256) void zero_f32_kernel(float4 *p, size_t n4)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256)
        p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

hipError_t launch_zero_f32(float *p, size_t n, hipStream_t st, const KernelTimer *tm)
{
    if (n == 0) return hipSuccess;
    const size_t n4 = n / 4;  // callers pass multiples of 4
    const int blocks = (int)((n4 + 255) / 256 < 2048 ? (n4 + 255) / 256 : 2048);
    launch_k(tm, LORA_K_ZERO, zero_f32_kernel, dim3(blocks), dim3(256), st, reinterpret_cast<float4 *>(p), n4);
    return hipGetLastError();
}

// k ranges are multiples of 512 elements: four wavefronts x one 128-element step.
static int shrink_k_len(int h_in, int want)
{
    int k_len = (h_in + want - 1) / want;
    return (k_len + 511) / 512 * 512;
}

int mfma_shrink_splits(int h_in, int want)
{
    if (want < 1) want = 1;
    const int k_len = shrink_k_len(h_in, want);
    return (h_in + k_len - 1) / k_len;
}

hipError_t launch_mfma_shrink(const ApplyArgs &a, const DevItem *tiles, int n_tiles, int k_splits, unsigned class_mask,
                              hipStream_t st, const KernelTimer *tm)
{
    if (n_tiles <= 0) return hipSuccess;
    const int k_len = shrink_k_len(a.h_in, k_splits < 1 ? 1 : k_splits);
    const int splits = (a.h_in + k_len - 1) / k_len;
    const dim3 grid(n_tiles, splits), block(256);
    const int at = splits > 1 ? 1 : 0;
    if (class_mask & 1u) launch_k(tm, LORA_K_MFMA_SHRINK, mfma_shrink_kernel<1, 128>, grid, block, st, a, tiles, k_len, at);
    if (class_mask & 2u) launch_k(tm, LORA_K_MFMA_SHRINK, mfma_shrink_kernel<2, 128>, grid, block, st, a, tiles, k_len, at);
    if (class_mask & 4u) launch_k(tm, LORA_K_MFMA_SHRINK, mfma_shrink_kernel<4, 64>, grid, block, st, a, tiles, k_len, at);
    if (class_mask & 8u) launch_k(tm, LORA_K_MFMA_SHRINK, mfma_shrink_kernel<8, 64>, grid, block, st, a, tiles, k_len, at);
    return hipGetLastError();
}

hipError_t launch_mfma_expand(const ApplyArgs &a, const DevItem *tiles, int n_tiles, hipStream_t st, const KernelTimer *tm)
{
    if (n_tiles <= 0) return hipSuccess;
    launch_k(tm, LORA_K_MFMA_EXPAND, mfma_expand_kernel, dim3(n_tiles, (a.h_out + EXPAND_COLS - 1) / EXPAND_COLS), dim3(256),
             st, a, tiles);
    return hipGetLastError();
}

}  // namespace lora
