/*
 * CPU ORACLE -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.
 *
 * Plain fp64 definition of the batched heterogeneous-rank LoRA apply that the
 * GPU library is checked against.  Only tests, the smoke check and the
 * benchmark's "cpu_baseline" leg may build or call this file; the GPU library
 * never does, and the two share no source.
 *
 * What is computed (paper section 3.1: per layer an adapter adds two matrix
 * products, A.x and B.(A.x), to the base product W.x, followed by an addition
 * that aggregates the results; section 2: requests that use different adapters
 * of different ranks share one batch).  Written in row-vector form, for every
 * token t that belongs to segment g with adapter i = seg_adapter[g] of rank r_i:
 *
 *     v[j]    = sum_k  x[t][k] * A_i[k][j]                 j < r_i   ("shrink")
 *     y[t][n] = base[t][n] + s_i * sum_j v[j] * B_i[j][n]  n < h_out ("expand" + add)
 *
 * with s_i = scale * alpha_i.  Tokens of a segment whose adapter index is
 * negative keep base[t][:] unchanged.  Everything is double; inputs arrive
 * already widened from whatever 16/32-bit format the caller stores them in.
 *
 * There is no blocking, no reordering and no layout trick here on purpose: the
 * loops are the definition.  The only concession to run time is an OpenMP
 * "parallel for" over tokens (tokens are independent), so that the benchmark
 * can time the oracle on all host cores.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Returns 0 on success, a negative number naming the first violated input rule. */
int oracle_lora_apply(
    int32_t T, int32_t h_in, int32_t h_out,
    const double *x,            /* [T][h_in]                                   */
    const double *base,         /* [T][h_out]  base-model output x.W            */
    double *y,                  /* [T][h_out]  result                           */
    int32_t n_seg,
    const int32_t *seg_offsets, /* [n_seg+1], seg_offsets[0]=0, [n_seg]=T, non-decreasing */
    const int32_t *seg_adapter, /* [n_seg] index into the arrays below, <0 = none */
    int32_t n_adapters,
    const int32_t *rank,        /* [n_adapters]                                 */
    const double *const *A,     /* A[i] -> [h_in][rank[i]] row-major            */
    const double *const *B,     /* B[i] -> [rank[i]][h_out] row-major           */
    const double *alpha,        /* [n_adapters]                                 */
    double scale)
{
    if (T < 0 || h_in <= 0 || h_out <= 0 || n_seg < 0) return -1;
    if (seg_offsets[0] != 0 || seg_offsets[n_seg] != T) return -2;
    for (int32_t g = 0; g < n_seg; ++g) {
        if (seg_offsets[g + 1] < seg_offsets[g]) return -3;
        if (seg_adapter[g] >= n_adapters) return -4;
    }

    /* token -> segment, by the dumbest possible loop */
    int32_t *tok_seg = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    if (!tok_seg) return -5;
    for (int32_t g = 0; g < n_seg; ++g)
        for (int32_t t = seg_offsets[g]; t < seg_offsets[g + 1]; ++t) tok_seg[t] = g;

    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t t = 0; t < T; ++t) {
        const int32_t i = seg_adapter[tok_seg[t]];
        const double *xt = x + (size_t)t * h_in;
        const double *bt = base + (size_t)t * h_out;
        double *yt = y + (size_t)t * h_out;
        if (i < 0) {
            for (int32_t n = 0; n < h_out; ++n) yt[n] = bt[n];
            continue;
        }
        const int32_t r = rank[i];
        const double s = scale * alpha[i];
        double *v = (double *)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
        if (!v) { fail = 1; continue; }
        for (int32_t j = 0; j < r; ++j) {
            double acc = 0.0;
            for (int32_t k = 0; k < h_in; ++k) acc += xt[k] * A[i][(size_t)k * r + j];
            v[j] = acc;
        }
        for (int32_t n = 0; n < h_out; ++n) {
            double acc = 0.0;
            for (int32_t j = 0; j < r; ++j) acc += v[j] * B[i][(size_t)j * h_out + n];
            yt[n] = bt[n] + s * acc;
        }
        free(v);
    }
    free(tok_seg);
    return fail ? -5 : 0;
}

/* Threads the parallel loop above runs on (1 when built without OpenMP). */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
