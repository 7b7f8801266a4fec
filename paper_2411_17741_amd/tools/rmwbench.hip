// Machine floors for the tile path on MI355X: a streaming read of 134 MB, the same read right
// after a kernel that wrote or read-modified-wrote another 134 MB (write-back still draining), and
// the read-modify-write itself.  Buffers rotate over 2 GiB so that nothing comes from the 256 MB
// Infinity Cache.  Each kernel is timed with its own start/stop events.
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 rmwbench.hip -o rmwbench && ./rmwbench
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("err %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)

__global__ __launch_bounds__(256) void rd(const uint4 *x, size_t n, unsigned *out)
{
    uint4 acc = make_uint4(0, 0, 0, 0);
    const size_t stride = (size_t)gridDim.x * 256 * 4;
    for (size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x; i < n; i += stride) {
        uint4 a = x[i], b = x[i + 256], c = x[i + 512], d = x[i + 768];
        acc.x ^= a.x ^ b.x ^ c.x ^ d.x; acc.y ^= a.y ^ b.y ^ c.y ^ d.y;
    }
    if ((acc.x ^ acc.y) == 0x12345u) out[0] = 1;
}
__global__ __launch_bounds__(256) void wr(uint4 *y, size_t n)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) y[i] = make_uint4(i, 1, 2, 3);
}
__global__ __launch_bounds__(256) void rmw(uint4 *y, size_t n)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) { uint4 v = y[i]; v.x += 1; y[i] = v; }
}

int main()
{
    const size_t SZ = (size_t)16384 * 4096 * 2, n = SZ / 16;
    unsigned char *buf; unsigned *out;
    CK(hipMalloc(&buf, SZ * 16)); CK(hipMalloc(&out, 4)); CK(hipMemset(buf, 1, SZ * 16));
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    for (int mode = 0; mode < 4; ++mode) {  // 0: read only, 1: write then read, 2: rmw then read, 3: time the rmw after a read
        double tot = 0; int cnt = 0;
        for (int i = 0; i < 40; ++i) {
            const uint4 *x = (const uint4 *)(buf + (size_t)(i & 7) * SZ);
            uint4 *y = (uint4 *)(buf + (size_t)(8 + (i & 7)) * SZ);
            if (mode == 1) wr<<<2048, 256>>>(y, n);
            if (mode == 2) rmw<<<2048, 256>>>(y, n);
            if (mode == 3) {
                rd<<<2048, 256>>>(x, n, out);
                hipExtLaunchKernelGGL(rmw, dim3(2048), dim3(256), 0, 0, e0, e1, 0, y, n);
            } else {
                hipExtLaunchKernelGGL(rd, dim3(2048), dim3(256), 0, 0, e0, e1, 0, x, n, out);
            }
            CK(hipEventSynchronize(e1));
            float ms; CK(hipEventElapsedTime(&ms, e0, e1));
            if (i >= 8) { tot += ms; ++cnt; }
        }
        printf("mode %d: timed kernel %.2f us (134 MB)\n", mode, tot / cnt * 1e3);
    }
    return 0;
}
