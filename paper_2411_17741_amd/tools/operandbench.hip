// Cost of MFMA-operand-shaped loads out of L2/L1 by lane mapping (microbenchmark).
// Every wavefront walks k over a 128-row x 8 KB matrix (1 MB, shared by all blocks: cache-resident), 16 rows x 64 B
// per instruction, with three lane mappings of the same bytes.
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 operandbench.hip -o operandbench && ./operandbench
#include <hip/hip_runtime.h>
#include <cstdio>
#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("hip error %s at %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)

template <int MODE>
__global__ __launch_bounds__(256) void oload(const char *__restrict__ at, int iters, uint4 *sink)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int row, piece;
    if (MODE == 0) { row = lane & 15; piece = lane >> 4; }        // operand layout: neighbours are different rows
    else if (MODE == 1) { row = lane >> 2; piece = lane & 3; }    // 4 neighbours share a row: 64 contiguous bytes
    else { row = (lane >> 4) * 4; piece = lane & 15; }            // 16 neighbours share a row: 256 contiguous bytes, 4 rows
    const char *p = at + (size_t)(16 * w + row) * 8192 + piece * 16;
    uint4 acc = make_uint4(0, 0, 0, 0);
    const int step = MODE == 2 ? 256 : 64;
    for (int it = 0; it < iters; ++it) {
        uint4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = *reinterpret_cast<const uint4 *>(p + (size_t)((it * 8 + j) * step % 8192) + (size_t)(j & 1) * 64 * 8192);
#pragma unroll
        for (int j = 0; j < 8; ++j) { acc.x ^= v[j].x; acc.y ^= v[j].y; acc.z ^= v[j].z; acc.w ^= v[j].w; }
    }
    if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u) sink[0] = acc;
}

int main()
{
    char *at; uint4 *sink;
    CHECK(hipMalloc(&at, 128 * 8192 + 4096));
    CHECK(hipMalloc(&sink, 64));
    CHECK(hipMemset(at, 1, 128 * 8192 + 4096));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    const int iters = 400, blocks = 512;
    auto run = [&](const char *name, auto kernel) -> int {
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(256), 0, 0, at, iters, sink);
        CHECK(hipDeviceSynchronize());
        CHECK(hipEventRecord(e0, 0));
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(256), 0, 0, at, iters, sink);
        CHECK(hipEventRecord(e1, 0));
        CHECK(hipEventSynchronize(e1));
        float ms = 0; CHECK(hipEventElapsedTime(&ms, e0, e1));
        const double loads_per_cu = 8.0 * iters * 8;  // 8 wavefronts per CU
        printf("%-58s %7.1f us  %6.1f ns per load instruction per CU  %5.2f TB/s\n", name, ms * 1e3, ms * 1e6 / loads_per_cu,
               (double)blocks * 4 * iters * 8 * 1024 / (ms * 1e-3) / 1e12);
        return 0;
    };
    if (run("16 rows x 4 pieces, neighbours in different rows", oload<0>)) return 1;
    if (run("16 rows x 4 pieces, 4 neighbours per row (64 B)", oload<1>)) return 1;
    if (run("4 rows x 16 pieces, 16 neighbours per row (256 B)", oload<2>)) return 1;
    return 0;
}
