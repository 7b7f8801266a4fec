// GEMV path of the batched LoRA apply for gfx950: tokens whose slot has only a few tokens in
// the batch (decode requests, short prompts).  Both kernels are bandwidth-bound streams of
// the slot's slab; every slab byte is read once per group of tokens that share the slot.
//
//   shrink:  v[t][j] = sum_k x[t][k] * A[k][j]        one wavefront per rank row j of At
//   expand:  y[t][n] += s * sum_j v[t][j] * B[j][n]   one lane per output column n of Bp
//
// (paper section 3.1: the two adapter products and the aggregation into the base output.)
#include "lora_device.h"

namespace lora {

// ---------------------------------------------------------------------------------------
// shrink.  Block = 4 wavefronts = up to 4 consecutive rank rows of one group.  A wavefront
// keeps U chunks (8 elements each) of its row per lane in registers, i.e. a K block of
// U*512 elements, while the block stages the same K block of up to TB token rows of x in
// LDS; every wavefront then forms its dot products against the staged rows and the partial
// sums are reduced across the 64 lanes at the end.
// ---------------------------------------------------------------------------------------
template <typename E, int U>
__global__ __launch_bounds__(256) void gemv_shrink_kernel(ApplyArgs a, const lora_item_t *__restrict__ items)
{
    constexpr int KB = U * 512;
    constexpr int TB = 4;
    __shared__ __attribute__((aligned(16))) E xs[TB * KB];

    const lora_item_t it = items[blockIdx.x];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const E *At = reinterpret_cast<const E *>(a.layer_base + a.slot_off[it.slot]);
    const bool row_ok = w < it.b;
    const int j = it.a + w;
    const E *arow = At + (size_t)j * a.h_in;
    const E *x = static_cast<const E *>(a.x);

    for (int t0 = 0; t0 < it.n_tok; t0 += TB) {
        const int nb = min(TB, it.n_tok - t0);
        float acc[TB];
#pragma unroll
        for (int t = 0; t < TB; ++t) acc[t] = 0.f;

        for (int k0 = 0; k0 < a.h_in; k0 += KB) {
            Chunk<E> av[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = k0 + (u * 64 + lane) * 8;
                if (row_ok && k < a.h_in) av[u] = load_chunk(arow + k);
                else av[u] = zero_chunk<E>();
            }
            __syncthreads();  // everyone is done reading the previous K block
            for (int t = 0; t < nb; ++t) {
                const E *xr = x + (size_t)a.tok_list[it.tok_off + t0 + t] * a.h_in;
                for (int c = threadIdx.x; c < KB / 8; c += 256) {
                    const int k = k0 + c * 8;
                    store_chunk(&xs[t * KB + c * 8], k < a.h_in ? load_chunk(xr + k) : zero_chunk<E>());
                }
            }
            __syncthreads();
#pragma unroll
            for (int t = 0; t < TB; ++t) {
                if (t < nb) {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const Chunk<E> xv = load_chunk(&xs[t * KB + (u * 64 + lane) * 8]);
                        acc[t] += dot_chunk(av[u], xv);
                    }
                }
            }
        }
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            if (t < nb) {
                const float s = wave_sum(acc[t]);
                if (lane == 0 && row_ok) a.v[(size_t)a.tok_list[it.tok_off + t0 + t] * a.v_stride + j] = s;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// expand.  Block = one wavefront = a run of output columns of one group.  A lane owns one
// column per pass; per granule of 8 ranks it reads the 8 B values of its column with one
// chunk load (the wavefront reads 64 consecutive chunks) and multiplies them with the
// scaled v of up to TB tokens, broadcast from LDS.
// ---------------------------------------------------------------------------------------
template <typename E>
__global__ __launch_bounds__(64) void gemv_expand_kernel(ApplyArgs a, const lora_item_t *__restrict__ items)
{
    constexpr int TB = 4;
    __shared__ __attribute__((aligned(16))) float vs[TB][LORA_MAX_RANK];

    const lora_item_t it = items[blockIdx.x];
    const int c0 = blockIdx.y * 1024 + it.a;
    if (c0 >= a.h_out) return;
    const int c1 = min(min(c0 + it.b, (int)(blockIdx.y + 1) * 1024), a.h_out);
    const int lane = threadIdx.x;
    const int rs = rank_storage(it.rank), rs8 = rs >> 3;
    const E *Bp = reinterpret_cast<const E *>(a.layer_base + a.slot_off[it.slot]) + (size_t)rs * a.h_in;
    const float s = a.scale * __int_as_float(it.c);
    E *y = static_cast<E *>(a.y);

    for (int t0 = 0; t0 < it.n_tok; t0 += TB) {
        const int nb = min(TB, it.n_tok - t0);
        __syncthreads();
        for (int t = 0; t < nb; ++t) {
            const float *vr = a.v + (size_t)a.tok_list[it.tok_off + t0 + t] * a.v_stride;
            for (int jj = lane; jj < rs; jj += 64) vs[t][jj] = jj < it.rank ? s * vr[jj] : 0.f;
        }
        __syncthreads();
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
                    if (t < nb) {
                        const float4 v0 = *reinterpret_cast<const float4 *>(&vs[t][j8 * 8]);
                        const float4 v1 = *reinterpret_cast<const float4 *>(&vs[t][j8 * 8 + 4]);
                        acc[t] += v0.x * bf[0] + v0.y * bf[1] + v0.z * bf[2] + v0.w * bf[3] + v1.x * bf[4] +
                                  v1.y * bf[5] + v1.z * bf[6] + v1.w * bf[7];
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < TB; ++t) {
                if (t < nb) {
                    E *yp = y + (size_t)a.tok_list[it.tok_off + t0 + t] * a.h_out + n;
                    *yp = from_float<E>(to_float(*yp) + acc[t]);
                }
            }
        }
    }
}

hipError_t launch_gemv_shrink(int dtype, const ApplyArgs &a, const lora_item_t *items, int n_items, hipStream_t st)
{
    if (n_items <= 0) return hipSuccess;
    if (dtype == LORA_BF16)
        hipLaunchKernelGGL((gemv_shrink_kernel<__bf16, 8>), dim3(n_items), dim3(256), 0, st, a, items);
    else
        hipLaunchKernelGGL((gemv_shrink_kernel<float, 4>), dim3(n_items), dim3(256), 0, st, a, items);
    return hipGetLastError();
}

hipError_t launch_gemv_expand(int dtype, const ApplyArgs &a, const lora_item_t *items, int n_items, hipStream_t st)
{
    if (n_items <= 0) return hipSuccess;
    const dim3 grid(n_items, (a.h_out + 1023) / 1024);
    if (dtype == LORA_BF16)
        hipLaunchKernelGGL((gemv_expand_kernel<__bf16>), grid, dim3(64), 0, st, a, items);
    else
        hipLaunchKernelGGL((gemv_expand_kernel<float>), grid, dim3(64), 0, st, a, items);
    return hipGetLastError();
}

}  // namespace lora
