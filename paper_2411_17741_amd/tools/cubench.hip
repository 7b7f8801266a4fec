// Issue rate of the two bf16 MFMA forms and of MFMA-operand reads from LDS on MI355X (microbenchmark):
// a loop of independent accumulations per wavefront, and the tile kernels' ds_read_b128 pattern (16 rows x
// 64 bytes per instruction) at several row pitches, with one block (one wavefront per SIMD) and with 512.
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 cubench.hip -o cubench && ./cubench
#include <hip/hip_runtime.h>
#include <cstdio>
#include <vector>
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("hip error %s at %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)

template <int NACC>
__global__ __launch_bounds__(256) void mfma_rate(float *out, int iters)
{
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(threadIdx.x * 0.001f + i); b[i] = (__bf16)(i * 0.5f); }
    floatx4 acc[NACC];
    for (int q = 0; q < NACC; ++q) acc[q] = floatx4{0.f, 0.f, 0.f, 0.f};
    long long t0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int q = 0; q < NACC; ++q) acc[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[q], 0, 0, 0);
    }
    float s = 0.f;
    for (int q = 0; q < NACC; ++q) s += acc[q][0] + acc[q][3];
    asm volatile("" ::"v"(s));
    long long t1 = __builtin_readcyclecounter();
    if (threadIdx.x == 0) { out[blockIdx.x * 2] = (float)(t1 - t0); out[blockIdx.x * 2 + 1] = s; }
}

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
template <int NACC>
__global__ __launch_bounds__(256) void mfma32_rate(float *out, int iters)
{
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(threadIdx.x * 0.001f + i); b[i] = (__bf16)(i * 0.5f); }
    floatx16 acc[NACC];
    for (int q = 0; q < NACC; ++q) for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;
    long long t0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int q = 0; q < NACC; ++q) acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[q], 0, 0, 0);
    }
    float s = 0.f;
    for (int q = 0; q < NACC; ++q) s += acc[q][0] + acc[q][15];
    asm volatile("" ::"v"(s));
    long long t1 = __builtin_readcyclecounter();
    if (threadIdx.x == 0) { out[blockIdx.x * 2] = (float)(t1 - t0); out[blockIdx.x * 2 + 1] = s; }
}

// every wavefront reads `n_rd` 16-byte operands per iteration with the tile kernels' pattern:
// lane (m = lane%16, g = lane/16) reads row m, piece 4*ks+g, rows `pitch` bytes apart
__global__ __launch_bounds__(256) void lds_rate(float *out, int iters, int pitch, int swz)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, m = lane & 15, g = lane >> 4;
    for (int i = tid; i < 64 * pitch / 4; i += 256) reinterpret_cast<float *>(lds)[i] = (float)i;
    __syncthreads();
    float s = 0.f;
    long long t0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int piece = ((4 * ks + g) ^ (swz ? (m & swz) : 0)) ^ (it & 1);
                const float4 v = *reinterpret_cast<const float4 *>(&lds[(16 * mb + m) * pitch + piece * 16]);
                s += v.x + v.w;
            }
    }
    asm volatile("" ::"v"(s));
    long long t1 = __builtin_readcyclecounter();
    if (lane == 0) { out[(blockIdx.x * 4 + (tid >> 6)) * 2] = (float)(t1 - t0); out[(blockIdx.x * 4 + (tid >> 6)) * 2 + 1] = s; }
}

int main()
{
    float *out;
    CHECK(hipMalloc(&out, 1 << 20));
    std::vector<float> h(1 << 18);
    const int iters = 2000;
    auto report = [&](const char *what, int n_blocks, int per_iter) {
        hipDeviceSynchronize();
        hipMemcpy(h.data(), out, n_blocks * 4 * 2 * sizeof(float), hipMemcpyDeviceToHost);
        printf("%-60s %8.1f cycles per instruction (per wavefront)\n", what, h[0] / ((double)iters * per_iter));
    };
    // MFMA: 1 block of 256 threads = 1 wavefront per SIMD; 512 blocks -> 2 per CU = 2 wavefronts per SIMD
    for (int blocks : {1, 512}) {
        hipLaunchKernelGGL(mfma_rate<4>, dim3(blocks), dim3(256), 0, 0, out, iters);
        CHECK(hipGetLastError());
        char buf[128]; snprintf(buf, sizeof buf, "mfma 16x16x32 bf16, 4 independent accumulators, %d block(s)", blocks);
        report(buf, blocks, 4);
        hipLaunchKernelGGL(mfma_rate<8>, dim3(blocks), dim3(256), 0, 0, out, iters);
        CHECK(hipGetLastError());
        snprintf(buf, sizeof buf, "mfma 16x16x32 bf16, 8 independent accumulators, %d block(s)", blocks);
        report(buf, blocks, 8);
    }
    for (int blocks : {1, 512}) {
        hipLaunchKernelGGL(mfma32_rate<4>, dim3(blocks), dim3(256), 0, 0, out, iters);
        CHECK(hipGetLastError());
        char buf[128]; snprintf(buf, sizeof buf, "mfma 32x32x16 bf16, 4 independent accumulators, %d block(s)", blocks);
        report(buf, blocks, 4);
    }
    {   // ticks of the cycle counter per microsecond: a long launch between two events
        hipEvent_t e0, e1;
        CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
        const int long_iters = 100000;
        CHECK(hipEventRecord(e0, 0));
        hipLaunchKernelGGL(mfma_rate<8>, dim3(512), dim3(256), 0, 0, out, long_iters);
        CHECK(hipEventRecord(e1, 0));
        CHECK(hipEventSynchronize(e1));
        float ms = 0; CHECK(hipEventElapsedTime(&ms, e0, e1));
        hipMemcpy(h.data(), out, 8 * sizeof(float), hipMemcpyDeviceToHost);
        printf("cycle counter: %.0f ticks in %.3f ms -> %.1f ticks per us; %d x 8 MFMAs per wavefront -> %.1f ns per MFMA per wavefront\n", h[0], ms, h[0] / (ms * 1e3), long_iters, ms * 1e6 / (8.0 * long_iters));
    }
    for (int pitch : {272, 288, 320, 256}) {
        for (int swz : {0, 15, 3}) {
            if (swz && pitch != 256) continue;
            for (int blocks : {1, 512}) {
                hipLaunchKernelGGL(lds_rate, dim3(blocks), dim3(256), 64 * pitch, 0, out, iters, pitch, swz);
                CHECK(hipGetLastError());
                char buf[128]; snprintf(buf, sizeof buf, "ds_read_b128 operand pattern, pitch %d swizzle %d, %d block(s)", pitch, swz, blocks);
                report(buf, blocks, 16);
            }
        }
    }
    hipFree(out);
    return 0;
}
