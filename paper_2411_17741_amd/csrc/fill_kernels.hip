// Repack of one freshly copied adapter part into the pool's slab layout (gfx950).
// The cache manager's "load a missing adapter from host memory" (paper section 4.2) hands
// over A [h_in][r] and B [r][h_out] in their mathematical row-major form; the apply kernels
// want At [rs][h_in] (rank-major) and Bp [rs/8][h_out][8] (rank-packed), rows r..rs-1 zero.
#include <algorithm>

#include "lora_device.h"

namespace lora {

constexpr int REPACK_HOST_BLOCKS = 32;

// One launch per part; the grid walks over the part's work units: units [0, h_in/64) transpose
// A, the rest pack B.  A fill runs beside the applies and slows them down for as long as its
// kernel is running, so from device memory (a staging buffer) the launch is one block per unit
// and over in a few microseconds; from host memory a few dozen blocks already keep more bytes in
// flight than the link needs and more would only hold wavefront slots.  The source may be
// device memory (a staging buffer) or pinned host memory read over PCIe, so it is read exactly
// once, in 16-byte pieces of contiguous runs, with every load of a thread issued before the
// first is used.
//
// A block: 64 rows k of A = one contiguous run of 64*r elements -> LDS -> At[j][k0 .. k0+63]
// for every stored rank j, written as 16-byte pieces along k.
// B block: 256 threads x 8 columns; a thread loads the 8 columns of the 8 ranks of a granule
// (8 loads, each 1 KB contiguous across a wavefront), transposes them in registers and writes
// 8 chunks of Bp = 128 contiguous bytes.
constexpr int REPACK_TROW = LORA_MAX_RANK + 2;  // LDS row stride in elements (breaks the power of two)

// one work unit of a part; every thread of the block calls it with the same arguments
template <typename E>
__device__ __forceinline__ void repack_unit(const E *__restrict__ A, const E *__restrict__ B, E *__restrict__ At, E *__restrict__ Bp,
                                            int h_in, int h_out, int r, int rs, int n_a_blocks, int unit, E *tile)
{
    constexpr int EPV = 16 / sizeof(E);            // elements per 16-byte piece
    constexpr int TROW = REPACK_TROW;
    const int tid = threadIdx.x;
    const int nb = (h_out + 256 * 8 - 1) / (256 * 8);
    {
        if (unit < n_a_blocks) {
            const int k0 = unit * 64;
            const uint4 *src = reinterpret_cast<const uint4 *>(A + (size_t)k0 * r);
            const int n_piece = 64 * r / EPV;              // 64 * r elements, a multiple of EPV
            constexpr int MAXP = 64 * LORA_MAX_RANK / EPV / 256;  // pieces per thread at most
            uint4 buf[MAXP];
#pragma unroll
            for (int it = 0; it < MAXP; ++it) {
                const int q = tid + 256 * it;
                buf[it] = src[q < n_piece ? q : 0];
            }
#pragma unroll
            for (int it = 0; it < MAXP; ++it) {
                const int q = tid + 256 * it;
                if (q < n_piece) {
                    const E *e = reinterpret_cast<const E *>(&buf[it]);
                    int kk = (q * EPV) / r, jj = (q * EPV) - kk * r;
#pragma unroll
                    for (int i = 0; i < EPV; ++i) {
                        tile[kk * TROW + jj] = e[i];
                        if (++jj == r) { jj = 0; ++kk; }
                    }
                }
            }
            __syncthreads();
            // At[j][k0 + 8*kq .. +7]: thread = (j, kq), 64 / EPV pieces per rank row
            constexpr int PPR = 64 / EPV;
            for (int idx = tid; idx < rs * PPR; idx += 256) {
                const int j = idx / PPR, kq = idx - j * PPR;
                E out[EPV];
#pragma unroll
                for (int i = 0; i < EPV; ++i) out[i] = j < r ? tile[(kq * EPV + i) * TROW + j] : from_float<E>(0.f);
                *reinterpret_cast<uint4 *>(At + (size_t)j * h_in + k0 + kq * EPV) = *reinterpret_cast<const uint4 *>(out);
            }
            __syncthreads();  // the next unit of this block overwrites the tile
        } else {
            // columns n0 .. n0+7 of granule j8
            const int bb = unit - n_a_blocks;
            const int j8 = bb / nb, n0 = ((bb - j8 * nb) * 256 + tid) * 8;
            if (n0 >= h_out) return;  // h_out is a multiple of 64, so a thread's 8 columns are all in or all out
            E in[8][8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int j = min(j8 * 8 + e, r - 1);
                const E *row = B + (size_t)j * h_out + n0;
                if constexpr (sizeof(E) == 2) {
                    *reinterpret_cast<uint4 *>(in[e]) = *reinterpret_cast<const uint4 *>(row);
                } else {
                    *reinterpret_cast<uint4 *>(in[e]) = *reinterpret_cast<const uint4 *>(row);
                    *reinterpret_cast<uint4 *>(in[e] + 4) = *reinterpret_cast<const uint4 *>(row + 4);
                }
            }
            E *o = Bp + ((size_t)j8 * h_out + n0) * 8;
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                E chunk[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) chunk[e] = j8 * 8 + e < r ? in[e][c] : from_float<E>(0.f);
                if constexpr (sizeof(E) == 2) {
                    *reinterpret_cast<uint4 *>(o + c * 8) = *reinterpret_cast<const uint4 *>(chunk);
                } else {
                    *reinterpret_cast<uint4 *>(o + c * 8) = *reinterpret_cast<const uint4 *>(chunk);
                    *reinterpret_cast<uint4 *>(o + c * 8 + 4) = *reinterpret_cast<const uint4 *>(chunk + 4);
                }
            }
        }
    }
}

template <typename E>
__global__ __launch_bounds__(256) void repack_kernel(const E *__restrict__ A, const E *__restrict__ B, E *__restrict__ At,
                                                     E *__restrict__ Bp, int h_in, int h_out, int r, int rs, int n_a_blocks)
{
    __shared__ E tile[64 * REPACK_TROW];
    const int n_units = n_a_blocks + (rs / 8) * ((h_out + 256 * 8 - 1) / (256 * 8));
    for (int unit = blockIdx.x; unit < n_units; unit += gridDim.x)  // uniform over the block
        repack_unit<E>(A, B, At, Bp, h_in, h_out, r, rs, n_a_blocks, unit, tile);
}

// Several parts of one adapter (same rank) in one launch: the blocks walk over the units of all parts.
template <typename E>
__global__ __launch_bounds__(256) void repack_parts_kernel(RepackTable t)
{
    __shared__ E tile[64 * REPACK_TROW];
    const int total = t.p[t.n - 1].unit_end;
    int part = 0;
    for (int g = blockIdx.x; g < total; g += gridDim.x) {  // uniform over the block; g only grows
        while (g >= t.p[part].unit_end) ++part;
        const RepackPart &q = t.p[part];
        const int first = part ? t.p[part - 1].unit_end : 0;
        E *At = static_cast<E *>(q.slab);
        repack_unit<E>(static_cast<const E *>(q.A), static_cast<const E *>(q.B), At, At + (size_t)t.rs * q.h_in, q.h_in, q.h_out, t.r,
                       t.rs, q.h_in / 64, g - first, tile);
    }
}

template <typename E>
static hipError_t repack_t(const void *sa, const void *sb, void *slab, int h_in, int h_out, int r, bool from_host, hipStream_t st)
{
    const int rs = rank_storage(r);
    E *At = static_cast<E *>(slab);
    E *Bp = At + (size_t)rs * h_in;
    const int n_a = h_in / 64, n_b = (rs / 8) * ((h_out + 2047) / 2048);
    hipLaunchKernelGGL((repack_kernel<E>), dim3(from_host ? std::min(n_a + n_b, REPACK_HOST_BLOCKS) : n_a + n_b), dim3(256), 0, st, static_cast<const E *>(sa),
                       static_cast<const E *>(sb), At, Bp, h_in, h_out, r, rs, n_a);
    return hipGetLastError();
}

// Sources must be 16-byte aligned (device staging buffers and pinned allocations are).
hipError_t launch_repack(int dtype, const void *src_A, const void *src_B, void *slab, int32_t h_in, int32_t h_out,
                         int32_t rank, bool from_host, hipStream_t st)
{
    if (dtype == LORA_BF16) return repack_t<__bf16>(src_A, src_B, slab, h_in, h_out, rank, from_host, st);
    return repack_t<float>(src_A, src_B, slab, h_in, h_out, rank, from_host, st);
}

// Parts of one adapter of rank `rank`: sources A, B and destination slab per part, all 16-byte aligned;
// unit_end is filled in here.  from_host as above.
hipError_t launch_repack_parts(int dtype, RepackTable &t, int32_t rank, bool from_host, hipStream_t st)
{
    if (t.n <= 0) return hipSuccess;
    t.r = rank;
    t.rs = rank_storage(rank);
    int total = 0;
    for (int i = 0; i < t.n; ++i) {
        total += t.p[i].h_in / 64 + (t.rs / 8) * ((t.p[i].h_out + 2047) / 2048);
        t.p[i].unit_end = total;
    }
    const dim3 grid(from_host ? std::min(total, 2 * REPACK_HOST_BLOCKS) : total);
    if (dtype == LORA_BF16) hipLaunchKernelGGL((repack_parts_kernel<__bf16>), grid, dim3(256), 0, st, t);
    else hipLaunchKernelGGL((repack_parts_kernel<float>), grid, dim3(256), 0, st, t);
    return hipGetLastError();
}

}  // namespace lora
