// What rate can the x stream of the tile shrink reach, by access pattern?  (microbenchmark)
// A block owns R token rows (8 KB apart) and walks its k range in steps of P bytes per row, with D steps in
// flight; nothing is computed.  T = 16384 rows of 8 KB (134 MB), buffers rotated (4 copies).  With ROT every
// block starts its walk at a different step (as the shrink kernel does): blocks that start together and step
// together otherwise all pull the same column window, rows 8 KB apart, which falls on few memory channels.
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 xwalkbench.hip -o xwalkbench && ./xwalkbench
#include <hip/hip_runtime.h>
#include <cstdio>
#include <vector>
#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("hip error %s at %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)

template <int R, int P, int D, bool ROT>
__global__ __launch_bounds__(256) void walk(const uint4 *__restrict__ x, int row_bytes, int k_bytes_per_block, int splits, uint4 *sink)
{
    constexpr int PER_STEP = R * P / 16;      // 16-byte pieces per step
    constexpr int NL = PER_STEP / 256;        // loads per thread per step
    static_assert(PER_STEP % 256 == 0, "");
    constexpr int PP = P / 16;                // pieces per row per step
    const int tile = blockIdx.x / splits, split = blockIdx.x % splits;
    const char *base = reinterpret_cast<const char *>(x) + (size_t)tile * R * row_bytes + (size_t)split * k_bytes_per_block;
    const int n_steps = k_bytes_per_block / P;
    const int phase = ROT ? (int)((blockIdx.x * 5u) % (unsigned)n_steps) : 0;
    auto at = [&](int st) { int s = min(st, n_steps - 1) + phase; s -= s >= n_steps ? n_steps : 0; return (size_t)s * P; };
    const char *src[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int idx = threadIdx.x + 256 * i;
        src[i] = base + (size_t)(idx / PP) * row_bytes + (idx % PP) * 16;
    }
    uint4 buf[D][NL];
    uint4 acc = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int d = 0; d < D; ++d)
#pragma unroll
        for (int i = 0; i < NL; ++i) buf[d][i] = *reinterpret_cast<const uint4 *>(src[i] + at(d));
    for (int st = 0; st < n_steps; st += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
#pragma unroll
            for (int i = 0; i < NL; ++i) { acc.x ^= buf[d][i].x; acc.y ^= buf[d][i].y; acc.z ^= buf[d][i].z; acc.w ^= buf[d][i].w; }
#pragma unroll
            for (int i = 0; i < NL; ++i) buf[d][i] = *reinterpret_cast<const uint4 *>(src[i] + at(st + d + D));
        }
    }
    if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u) sink[0] = acc;  // never true in practice: keeps the loads
}

int main()
{
    const int T = 16384, row_bytes = 8192, NBUF = 4;
    const size_t bytes = (size_t)T * row_bytes;
    uint4 *x, *sink;
    CHECK(hipMalloc(&x, bytes * NBUF));
    CHECK(hipMalloc(&sink, 64));
    CHECK(hipMemset(x, 1, bytes * NBUF));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    auto run = [&](const char *name, auto kernel, int R, int splits) -> int {
        const int blocks = T / R * splits, kb = row_bytes / splits;
        for (int it = 0; it < 3; ++it) hipLaunchKernelGGL(kernel, dim3(blocks), dim3(256), 0, 0, x + (size_t)(it % NBUF) * (bytes / 16), row_bytes, kb, splits, sink);
        CHECK(hipDeviceSynchronize());
        const int reps = 20;
        CHECK(hipEventRecord(e0, 0));
        for (int it = 0; it < reps; ++it) hipLaunchKernelGGL(kernel, dim3(blocks), dim3(256), 0, 0, x + (size_t)(it % NBUF) * (bytes / 16), row_bytes, kb, splits, sink);
        CHECK(hipEventRecord(e1, 0));
        CHECK(hipEventSynchronize(e1));
        float ms = 0; CHECK(hipEventElapsedTime(&ms, e0, e1));
        printf("%-58s blocks %5d  %7.1f us  %5.2f TB/s\n", name, blocks, ms * 1e3 / reps, bytes / (ms * 1e-3 / reps) / 1e12);
        return 0;
    };
    if (run("64 rows x 256 B, 3 in flight, 1 split(s)", walk<64, 256, 3, false>, 64, 1)) return 1;
    if (run("64 rows x 256 B, 3 in flight, 1 split(s), rotated start", walk<64, 256, 3, true>, 64, 1)) return 1;
    if (run("64 rows x 256 B, 3 in flight, 2 split(s)", walk<64, 256, 3, false>, 64, 2)) return 1;
    if (run("64 rows x 256 B, 3 in flight, 2 split(s), rotated start", walk<64, 256, 3, true>, 64, 2)) return 1;
    if (run("64 rows x 256 B, 3 in flight, 4 split(s)", walk<64, 256, 3, false>, 64, 4)) return 1;
    if (run("64 rows x 256 B, 3 in flight, 4 split(s), rotated start", walk<64, 256, 3, true>, 64, 4)) return 1;
    if (run("64 rows x 256 B, 1 in flight, 2 split(s)", walk<64, 256, 1, false>, 64, 2)) return 1;
    if (run("64 rows x 256 B, 1 in flight, 2 split(s), rotated start", walk<64, 256, 1, true>, 64, 2)) return 1;
    if (run("64 rows x 512 B, 2 in flight, 2 split(s)", walk<64, 512, 2, false>, 64, 2)) return 1;
    if (run("64 rows x 512 B, 2 in flight, 2 split(s), rotated start", walk<64, 512, 2, true>, 64, 2)) return 1;
    if (run("32 rows x 512 B, 3 in flight, 2 split(s)", walk<32, 512, 3, false>, 32, 2)) return 1;
    if (run("32 rows x 512 B, 3 in flight, 2 split(s), rotated start", walk<32, 512, 3, true>, 32, 2)) return 1;
    if (run("16 rows x 1024 B, 3 in flight, 1 split(s)", walk<16, 1024, 3, false>, 16, 1)) return 1;
    if (run("16 rows x 1024 B, 3 in flight, 1 split(s), rotated start", walk<16, 1024, 3, true>, 16, 1)) return 1;
    if (run("128 rows x 128 B, 3 in flight, 2 split(s)", walk<128, 128, 3, false>, 128, 2)) return 1;
    if (run("128 rows x 128 B, 3 in flight, 2 split(s), rotated start", walk<128, 128, 3, true>, 128, 2)) return 1;
    if (run("128 rows x 128 B, 3 in flight, 4 split(s)", walk<128, 128, 3, false>, 128, 4)) return 1;
    if (run("128 rows x 128 B, 3 in flight, 4 split(s), rotated start", walk<128, 128, 3, true>, 128, 4)) return 1;
    if (run("64 rows x 1024 B, 1 in flight, 2 split(s)", walk<64, 1024, 1, false>, 64, 2)) return 1;
    if (run("64 rows x 1024 B, 1 in flight, 2 split(s), rotated start", walk<64, 1024, 1, true>, 64, 2)) return 1;
    return 0;
}
