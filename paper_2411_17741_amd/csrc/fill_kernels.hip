// Repack of one freshly copied adapter part into the pool's slab layout (gfx950).
// The cache manager's "load a missing adapter from host memory" (paper section 4.2) hands
// over A [h_in][r] and B [r][h_out] in their mathematical row-major form; the apply kernels
// want At [rs][h_in] (rank-major) and Bp [rs/8][h_out][8] (rank-packed), rows r..rs-1 zero.
#include "lora_device.h"

namespace lora {

// At[j][k] = A[k][j].  A 64(k) x 8(j) patch per 256-thread block goes through LDS so that
// both the reads (along j, then k) and the writes (along k) are contiguous runs.
template <typename E>
__global__ __launch_bounds__(256) void repack_a_kernel(const E *__restrict__ A, E *__restrict__ At, int h_in, int r, int rs)
{
    __shared__ E tile[64][64 + 1];
    const int k0 = blockIdx.x * 64, j0 = blockIdx.y * 64;
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int kk = i >> 6, jj = i & 63;  // consecutive threads walk along j (contiguous in A)
        const int k = k0 + kk, j = j0 + jj;
        tile[kk][jj] = (k < h_in && j < r) ? A[(size_t)k * r + j] : from_float<E>(0.f);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int jj = i >> 6, kk = i & 63;  // consecutive threads walk along k (contiguous in At)
        const int k = k0 + kk, j = j0 + jj;
        if (k < h_in && j < rs) At[(size_t)j * h_in + k] = tile[kk][jj];
    }
}

// Bp[j/8][n][j%8] = B[j][n]: one thread per (granule, column), 8 strided reads (each
// contiguous across the threads of a wavefront), one contiguous 8-element write.
template <typename E>
__global__ __launch_bounds__(256) void repack_b_kernel(const E *__restrict__ B, E *__restrict__ Bp, int h_out, int r, int rs)
{
    const int n = blockIdx.x * 256 + threadIdx.x, j8 = blockIdx.y;
    if (n >= h_out) return;
    E *o = Bp + ((size_t)j8 * h_out + n) * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int j = j8 * 8 + e;
        o[e] = j < r ? B[(size_t)j * h_out + n] : from_float<E>(0.f);
    }
}

template <typename E>
static hipError_t repack_t(const void *sa, const void *sb, void *slab, int h_in, int h_out, int r, hipStream_t st)
{
    const int rs = rank_storage(r);
    E *At = static_cast<E *>(slab);
    E *Bp = At + (size_t)rs * h_in;
    hipLaunchKernelGGL((repack_a_kernel<E>), dim3((h_in + 63) / 64, (rs + 63) / 64), dim3(256), 0, st,
                       static_cast<const E *>(sa), At, h_in, r, rs);
    hipLaunchKernelGGL((repack_b_kernel<E>), dim3((h_out + 255) / 256, rs / 8), dim3(256), 0, st,
                       static_cast<const E *>(sb), Bp, h_out, r, rs);
    return hipGetLastError();
}

hipError_t launch_repack(int dtype, const void *stage_A, const void *stage_B, void *slab, int32_t h_in, int32_t h_out,
                         int32_t rank, hipStream_t st)
{
    if (dtype == LORA_BF16) return repack_t<__bf16>(stage_A, stage_B, slab, h_in, h_out, rank, st);
    return repack_t<float>(stage_A, stage_B, slab, h_in, h_out, rank, st);
}

}  // namespace lora
