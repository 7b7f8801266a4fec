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
constexpr int KT = 64;                 // shrink: k elements per LDS tile
constexpr int AT_ROW = KT * 2 + 16;    // bytes per At row in LDS (padded: rows land in distinct banks)
constexpr int VS_ROW = LORA_MAX_RANK * 2 + 16;  // bytes per token row of the staged V tile
constexpr int EXPAND_PASSES = 2;       // expand: column passes of 256 per block
}  // namespace

// ---------------------------------------------------------------------------------------
// shrink.  Block = 4 wavefronts; wavefront w owns tokens 16w..16w+15 of the tile and all
// rank blocks (up to 8 of 16 ranks).  x is loaded straight into A-operand registers (each x
// element is used by exactly one wavefront); the At tile is shared through LDS, double
// buffered, one barrier per K tile.  Lane group g covers k = kt + 16g .. +15 (32 contiguous
// bytes per lane), MFMA step i uses the i-th 8 of them.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void mfma_shrink_kernel(ApplyArgs a, const lora_item_t *__restrict__ tiles,
                                                          int k_len, int use_atomic)
{
    __shared__ __attribute__((aligned(16))) unsigned char at_lds[2][LORA_MAX_RANK * AT_ROW];

    const lora_item_t it = tiles[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int rs = rank_storage(it.rank);
    const int NB = (it.rank + 15) >> 4;
    const int k_begin = blockIdx.y * k_len;
    const int k_end = min(a.h_in, k_begin + k_len);
    const int n_kt = (k_end - k_begin + KT - 1) / KT;
    if (n_kt <= 0) return;

    const __bf16 *At = reinterpret_cast<const __bf16 *>(a.layer_base + a.slot_off[it.slot]);
    const __bf16 *x = static_cast<const __bf16 *>(a.x);

    const bool wave_live = 16 * w < it.n_tok;
    const int ti_a = 16 * w + m;  // token row this lane feeds as A operand
    const bool a_ok = ti_a < it.n_tok;
    const __bf16 *xrow = x + (size_t)(a_ok ? a.tok_list[it.tok_off + ti_a] : 0) * a.h_in + 16 * g;

    // At tile loader: 8 lanes per row (128 bytes), 32 rows per pass
    const int lp = tid & 7, lr = tid >> 3;
    const int n_pass = (16 * NB + 31) >> 5;

    uint4 xa[2], xn[2], tn[4];
    auto load_x = [&](int kt, uint4(&dst)[2]) {
        if (a_ok) {
            const uint4 *p = reinterpret_cast<const uint4 *>(xrow + kt);
            dst[0] = p[0];
            dst[1] = p[1];
        } else {
            dst[0] = dst[1] = make_uint4(0, 0, 0, 0);
        }
    };
    auto load_at = [&](int kt) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int row = p * 32 + lr;
            if (p < n_pass && row < rs)
                tn[p] = *reinterpret_cast<const uint4 *>(At + (size_t)row * a.h_in + kt + lp * 8);
            else
                tn[p] = make_uint4(0, 0, 0, 0);
        }
    };
    auto store_at = [&](int buf) {
#pragma unroll
        for (int p = 0; p < 4; ++p)
            if (p < n_pass) *reinterpret_cast<uint4 *>(&at_lds[buf][(p * 32 + lr) * AT_ROW + lp * 16]) = tn[p];
    };

    floatx4 acc[8];
#pragma unroll
    for (int nb = 0; nb < 8; ++nb) acc[nb] = floatx4{0.f, 0.f, 0.f, 0.f};

    load_x(k_begin, xa);
    load_at(k_begin);
    store_at(0);
    __syncthreads();

    for (int kt_i = 0; kt_i < n_kt; ++kt_i) {
        const int cur = kt_i & 1;
        const bool more = kt_i + 1 < n_kt;
        if (more) {
            load_x(k_begin + (kt_i + 1) * KT, xn);
            load_at(k_begin + (kt_i + 1) * KT);
        }
        if (wave_live) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const bf16x8 av = __builtin_bit_cast(bf16x8, xa[i]);
#pragma unroll
                for (int nb = 0; nb < 8; ++nb) {
                    if (nb < NB) {
                        const bf16x8 bv = *reinterpret_cast<const bf16x8 *>(
                            &at_lds[cur][(16 * nb + m) * AT_ROW + (16 * g + 8 * i) * 2]);
                        acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bv, acc[nb], 0, 0, 0);
                    }
                }
            }
        }
        if (more) {
            store_at(cur ^ 1);
            xa[0] = xn[0];
            xa[1] = xn[1];
        }
        __syncthreads();
    }

    if (!wave_live) return;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int ti = 16 * w + 4 * g + r;
        if (ti < it.n_tok) {
            float *vr = a.v + (size_t)a.tok_list[it.tok_off + ti] * a.v_stride;
#pragma unroll
            for (int nb = 0; nb < 8; ++nb) {
                const int jr = 16 * nb + m;
                if (nb < NB && jr < it.rank) {
                    if (use_atomic) unsafeAtomicAdd(vr + jr, acc[nb][r]);
                    else vr[jr] = acc[nb][r];
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// expand.  Block = 4 wavefronts, tile of up to 64 tokens x 256*EXPAND_PASSES columns.  The
// scaled V tile is staged once in LDS as bf16.  The product is formed transposed (rows =
// output columns, columns = tokens) so that a lane ends up with runs of 8 consecutive
// output columns of one token: block b of the 4 column blocks of a wavefront maps MFMA row
// 4q+r to column 8q + 4(b&1) + r + 32(b>>1), which makes the read-modify-write of base_out a
// pair of 16-byte accesses per lane, 64 contiguous bytes per token row across a lane group.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void mfma_expand_kernel(ApplyArgs a, const lora_item_t *__restrict__ tiles)
{
    __shared__ __attribute__((aligned(16))) unsigned char vs[LORA_TILE_TOKENS * VS_ROW];

    const lora_item_t it = tiles[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int rs8 = rank_storage(it.rank) >> 3;
    const int KS = (it.rank + 31) >> 5;  // MFMA k steps of 32 ranks
    const int c8 = KS * 4;               // staged chunks (8 ranks) per token
    const float s = a.scale * __int_as_float(it.c);
    const __bf16 *Bp = reinterpret_cast<const __bf16 *>(a.layer_base + a.slot_off[it.slot]) +
                       (size_t)rank_storage(it.rank) * a.h_in;
    __bf16 *y = static_cast<__bf16 *>(a.y);

    // stage s.V as bf16: vs[token][rank]
    for (int idx = tid; idx < LORA_TILE_TOKENS * c8; idx += 256) {
        const int ti = idx / c8, j8 = idx - ti * c8;
        bf16x8 o;
        if (ti < it.n_tok) {
            const float *vr = a.v + (size_t)a.tok_list[it.tok_off + ti] * a.v_stride + j8 * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (__bf16)((j8 * 8 + e < it.rank) ? s * vr[e] : 0.f);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (__bf16)0.f;
        }
        *reinterpret_cast<bf16x8 *>(&vs[ti * VS_ROW + j8 * 16]) = o;
    }
    __syncthreads();

    // token rows this lane reads/writes in the epilogue: 16*tb + m
    size_t yoff[4];
    bool yok[4];
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
        const int ti = 16 * tb + m;
        yok[tb] = ti < it.n_tok;
        yoff[tb] = yok[tb] ? (size_t)a.tok_list[it.tok_off + ti] * a.h_out : 0;
    }
    const int n_tb = (it.n_tok + 15) >> 4;

    for (int cp = 0; cp < EXPAND_PASSES; ++cp) {
        const int nw0 = (blockIdx.y * EXPAND_PASSES + cp) * 256 + 64 * w;
        if (nw0 >= a.h_out) break;

        uint4 yr[4][2];
#pragma unroll
        for (int tb = 0; tb < 4; ++tb)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                if (yok[tb]) yr[tb][h] = *reinterpret_cast<const uint4 *>(y + yoff[tb] + nw0 + 8 * g + 32 * h);

        floatx4 acc[4][4];
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int tb = 0; tb < 4; ++tb) acc[b][tb] = floatx4{0.f, 0.f, 0.f, 0.f};

        for (int ks = 0; ks < KS; ++ks) {
            const int j8 = 4 * ks + g;
            bf16x8 aop[4], bop[4];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int n = nw0 + 8 * (m >> 2) + 4 * (b & 1) + (m & 3) + 32 * (b >> 1);
                uint4 raw = make_uint4(0, 0, 0, 0);
                if (j8 < rs8) raw = *reinterpret_cast<const uint4 *>(Bp + ((size_t)j8 * a.h_out + n) * 8);
                aop[b] = __builtin_bit_cast(bf16x8, raw);
            }
#pragma unroll
            for (int tb = 0; tb < 4; ++tb)
                if (tb < n_tb) bop[tb] = *reinterpret_cast<const bf16x8 *>(&vs[(16 * tb + m) * VS_ROW + j8 * 16]);
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int tb = 0; tb < 4; ++tb)
                    if (tb < n_tb) acc[b][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop[b], bop[tb], acc[b][tb], 0, 0, 0);
        }

#pragma unroll
        for (int tb = 0; tb < 4; ++tb) {
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

hipError_t launch_zero_f32(float *p, size_t n, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    const size_t n4 = n / 4;  // callers pass multiples of 4
    const int blocks = (int)((n4 + 255) / 256 < 2048 ? (n4 + 255) / 256 : 2048);
    hipLaunchKernelGGL(zero_f32_kernel, dim3(blocks), dim3(256), 0, st, reinterpret_cast<float4 *>(p), n4);
    return hipGetLastError();
}

hipError_t launch_mfma_shrink(const ApplyArgs &a, const lora_item_t *tiles, int n_tiles, int k_splits, hipStream_t st)
{
    if (n_tiles <= 0) return hipSuccess;
    int k_len = (a.h_in + k_splits - 1) / k_splits;
    k_len = (k_len + KT - 1) / KT * KT;
    const int splits = (a.h_in + k_len - 1) / k_len;
    hipLaunchKernelGGL(mfma_shrink_kernel, dim3(n_tiles, splits), dim3(256), 0, st, a, tiles, k_len, splits > 1 ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_mfma_expand(const ApplyArgs &a, const lora_item_t *tiles, int n_tiles, hipStream_t st)
{
    if (n_tiles <= 0) return hipSuccess;
    const int cols_per_block = 256 * EXPAND_PASSES;
    hipLaunchKernelGGL(mfma_expand_kernel, dim3(n_tiles, (a.h_out + cols_per_block - 1) / cols_per_block), dim3(256), 0,
                       st, a, tiles);
    return hipGetLastError();
}

}  // namespace lora
