// GEMV path of the batched LoRA apply for gfx950: tokens whose slot has only a few tokens in
// the batch (decode requests, short prompts).  Both phases are bandwidth-bound streams of
// the slot's slab.  A work item is a batch of up to 4 tokens of one slot; every load an item
// needs -- slab, activations, intermediate -- is issued before the first one is used, so an
// item costs one trip to memory, and the batches of a popular slot run side by side (its slab
// then comes out of L2 for all but the first).
//
//   shrink:  v[t][j] = sum_k x[t][k] * A[k][j]        wavefronts own (parts of) rank rows of At
//   expand:  y[t][n] += s * sum_j v[t][j] * B[j][n]   lanes own output columns of Bp
//
// The two phases run as two launches.  A one-launch (fused) form, in which the expand wavefronts
// fetch their part of Bp and base_out while the shrink blocks are still working and then wait on
// a per-batch counter for the intermediate, is kept as an option: on this 8-XCD part the
// device-scope release/acquire it needs per wavefront costs more than the second launch.
//
// (paper section 3.1: the two adapter products and the aggregation into the base output.)
#include "lora_device.h"

namespace lora {

constexpr int TB = LORA_GEMV_BATCH;

// How the two phases hand over v.
struct Handover {
    int32_t *counters;  // nullptr: separate launches, the stream orders the phases
    int32_t epoch;      // applies of this plan so far, this one included
    int32_t *fault;
};

// ---------------------------------------------------------------------------------------
// shrink.  Block = 4 wavefronts working on R rank rows, W = 4/R wavefronts per row, each
// covering every W-th run of 64 chunks (8 elements each) of the row: 8 chunk loads per lane
// per pass.  x chunks of the item's tokens are read at the same offsets, straight from global
// memory (the wavefronts of a block read the same lines at the same time).  Partial sums are
// reduced over the 64 lanes and, for W > 1, over the W wavefronts through LDS.  A work item
// names 4 rows, so an item takes W blocks (`part` = which).
// ---------------------------------------------------------------------------------------
template <typename E, int R>
__device__ __forceinline__ void gemv_shrink_block(const ApplyArgs &a, const GemvItem &it, int part, const Handover &ho,
                                                  float (*red)[TB])
{
    constexpr int W = 4 / R;
    constexpr int U = 8;
    const int j0 = it.a & 0xff, n_rows = (it.a >> 8) & 0xf, batch = it.a >> 12;
    if (part * R >= n_rows) return;  // whole block has no row (uniform)
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int rr = part * R + w / W, kp = w % W;  // row inside the item, k part of this wavefront
    const bool row_ok = rr < n_rows;
    const int j = j0 + rr;
    const E *arow = reinterpret_cast<const E *>(a.proj_base + (int64_t)it.row * a.row_bytes) + (size_t)j * a.h_in;
    const E *x = static_cast<const E *>(a.x);
    const int n_chunks = a.h_in >> 3;

    float acc[TB];
#pragma unroll
    for (int t = 0; t < TB; ++t) acc[t] = 0.f;

    // Loads are unconditional (addresses clamped to something valid, results masked), so that
    // the compiler can issue all of them back to back and wait once.
    constexpr int TS = sizeof(E) == 2 ? TB : 2;  // tokens whose x chunks are in registers at once
    const E *arow_safe = row_ok ? arow : arow - (size_t)rr * a.h_in;  // the item's first row always exists
    for (int c0 = 0; c0 < n_chunks; c0 += W * 64 * U) {
        Chunk<E> av[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + (u * W + kp) * 64 + lane;
            av[u] = load_chunk(arow_safe + (size_t)min(c, n_chunks - 1) * 8);
        }
#pragma unroll
        for (int t0 = 0; t0 < TB; t0 += TS) {
            Chunk<E> xv[TS][U];
#pragma unroll
            for (int t = 0; t < TS; ++t) {
                const int tok = it.tok[t0 + t] >= 0 ? it.tok[t0 + t] : it.tok[0];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int c = c0 + (u * W + kp) * 64 + lane;
                    xv[t][u] = load_chunk(x + (size_t)tok * a.h_in + (size_t)min(c, n_chunks - 1) * 8);
                }
            }
#pragma unroll
            for (int t = 0; t < TS; ++t) {
                if (it.tok[t0 + t] >= 0) {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int cb = c0 + (u * W + kp) * 64;  // uniform over the wavefront
                        if (cb + 64 <= n_chunks) {
                            acc[t0 + t] = dot_chunk_acc(acc[t0 + t], av[u], xv[t][u]);
                        } else if (cb < n_chunks) {  // ragged end of the row: clamped lanes do not count
                            const float d = dot_chunk_acc(0.f, av[u], xv[t][u]);
                            acc[t0 + t] += cb + lane < n_chunks ? d : 0.f;
                        }
                    }
                }
            }
        }
    }
#pragma unroll
    for (int t = 0; t < TB; ++t)
        if (it.tok[t] >= 0) acc[t] = wave_sum(acc[t]);
    if (W > 1) {
        if (lane == 0) {
#pragma unroll
            for (int t = 0; t < TB; ++t) red[w][t] = acc[t];
        }
        __syncthreads();
        if (kp == 0) {
#pragma unroll
            for (int t = 0; t < TB; ++t) {
                float s = 0.f;
#pragma unroll
                for (int q = 0; q < W; ++q) s += red[w + q][t];
                acc[t] = s;
            }
        }
    }
    if (lane == 0 && kp == 0 && row_ok) {
        if (ho.counters) {
            // The waiting expand wavefronts may run on another XCD, whose L2 is not coherent with
            // this one: a device-scope release (L2 write-back) before the increment, a device-scope
            // acquire (L2 invalidate) after the wait.  Cheaper hand-overs (write-through stores and
            // loads without the cache maintenance) were tried and do return stale data.
#pragma unroll
            for (int t = 0; t < TB; ++t)
                if (it.tok[t] >= 0) a.v[(size_t)it.tok[t] * a.v_stride + j] = acc[t];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            __hip_atomic_fetch_add(&ho.counters[batch], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
#pragma unroll
            for (int t = 0; t < TB; ++t)
                if (it.tok[t] >= 0) a.v[(size_t)it.tok[t] * a.v_stride + j] = acc[t];
        }
    }
}

// Waits until all `rank` rows of the batch are there.  Bounded: a wavefront that gives up
// raises the fault flag and does no work.
__device__ __forceinline__ bool wait_for_batch(const Handover &ho, int batch, int rank)
{
    const int32_t target = ho.epoch * rank;
    for (int spin = 0; spin < (1 << 18); ++spin) {
        if (__hip_atomic_load(&ho.counters[batch], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target) {
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            return true;
        }
        __builtin_amdgcn_s_sleep(4);
    }
    if ((threadIdx.x & 63) == 0) __hip_atomic_store(ho.fault, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return false;
}

__device__ __forceinline__ float load_v(const Handover &, const float *p) { return *p; }

// ---------------------------------------------------------------------------------------
// expand, ranks whose storage is 8, 16, 32, 64 or 128 rows (RS8 = 1, 2, 4, 8, 16 granules).
// One wavefront per unit; a lane owns P = 16/RS8 output columns (n = c0 + lane + 64p) and
// loads all of its 16 chunks of Bp and the base_out values it will update up front, then the
// v of the item's tokens (one value per lane, broadcast with readlane when used).
// ---------------------------------------------------------------------------------------
template <typename E, int RS8>
__device__ __forceinline__ void gemv_expand_body(const ApplyArgs &a, const GemvItem &it, int c0, int c1, const E *Bp,
                                                 const Handover &ho)
{
    constexpr int P = 16 / RS8;
    const int lane = threadIdx.x & 63;
    const float s = a.scale * it.alpha;
    E *y = static_cast<E *>(a.y);

    // Loads are unconditional (columns and tokens clamped to valid ones, results discarded), so
    // that all of them are issued back to back; stores come after all the arithmetic.
    Chunk<E> b[P][RS8];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int n = c0 + lane + 64 * p;
        const int ns = n < c1 ? n : c0 + lane;
#pragma unroll
        for (int j8 = 0; j8 < RS8; ++j8) b[p][j8] = load_chunk(Bp + ((size_t)j8 * a.h_out + ns) * 8);
    }
    E yv[TB][P];
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        const int tok = it.tok[t] >= 0 ? it.tok[t] : it.tok[0];
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int n = c0 + lane + 64 * p;
            yv[t][p] = y[(size_t)tok * a.h_out + (n < c1 ? n : c0 + lane)];
        }
    }
    if (ho.counters && !wait_for_batch(ho, it.a >> 4, it.rank)) return;
    float vlo[TB], vhi[TB];
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        const int tok = it.tok[t] >= 0 ? it.tok[t] : it.tok[0];
        const float *vr = a.v + (size_t)tok * a.v_stride;  // rows are at least 128 floats long
        vlo[t] = load_v(ho, vr + lane);
        vhi[t] = RS8 > 8 ? load_v(ho, vr + lane + 64) : 0.f;
    }
    float acc[TB][P];
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        if (lane >= it.rank) vlo[t] = 0.f;  // what lies beyond the rank was never written
        if (lane + 64 >= it.rank) vhi[t] = 0.f;
#pragma unroll
        for (int p = 0; p < P; ++p) acc[t][p] = 0.f;
    }
#pragma unroll
    for (int j8 = 0; j8 < RS8; ++j8) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            float bf[8];
            unpack_chunk(b[p][j8], bf);
#pragma unroll
            for (int t = 0; t < TB; ++t) {
                if (it.tok[t] >= 0) {  // uniform
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int jj = j8 * 8 + i;
                        const float vj = __builtin_bit_cast(
                            float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, jj < 64 ? vlo[t] : vhi[t]), jj & 63));
                        acc[t][p] += vj * bf[i];
                    }
                }
            }
        }
    }
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        if (it.tok[t] >= 0) {
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const int n = c0 + lane + 64 * p;
                if (n < c1) y[(size_t)it.tok[t] * a.h_out + n] = from_float<E>(to_float(yv[t][p]) + s * acc[t][p]);
            }
        }
    }
}

// Any other rank: granule loop, v of the item's tokens staged in this wavefront's LDS rows.
template <typename E>
__device__ __forceinline__ void gemv_expand_generic(const ApplyArgs &a, const GemvItem &it, int c0, int c1, const E *Bp,
                                                    const Handover &ho, float (*vs)[LORA_MAX_RANK])
{
    const int lane = threadIdx.x & 63;
    const int rs = rank_storage(it.rank), rs8 = rs >> 3;
    const float s = a.scale * it.alpha;
    E *y = static_cast<E *>(a.y);
    if (ho.counters && !wait_for_batch(ho, it.a >> 4, it.rank)) return;
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        if (it.tok[t] >= 0) {
            const float *vr = a.v + (size_t)it.tok[t] * a.v_stride;
            for (int jj = lane; jj < rs; jj += 64) vs[t][jj] = jj < it.rank ? s * load_v(ho, vr + jj) : 0.f;
        }
    }
    // only this wavefront reads what it wrote, and a wavefront's LDS operations execute in order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
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
                if (it.tok[t] >= 0) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) acc[t] += vs[t][j8 * 8 + i] * bf[i];
                }
            }
        }
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            if (it.tok[t] >= 0) {
                E *yp = y + (size_t)it.tok[t] * a.h_out + n;
                *yp = from_float<E>(to_float(*yp) + acc[t]);
            }
        }
    }
}

// One expand unit = (item, 1024-column super-chunk `sc`), worked on by one wavefront.
template <typename E>
__device__ __forceinline__ void gemv_expand_wave(const ApplyArgs &a, const GemvItem &it, int sc, const Handover &ho,
                                                 float (*vs)[LORA_MAX_RANK])
{
    const int rs = rank_storage(it.rank);
    const int n_cols = 64 * max(1, 128 / rs);
    const int c0 = sc * 1024 + (it.a & 0xf) * 64;
    if (c0 >= a.h_out) return;
    const int c1 = min(min(c0 + n_cols, (sc + 1) * 1024), a.h_out);
    const E *Bp = reinterpret_cast<const E *>(a.proj_base + (int64_t)it.row * a.row_bytes) + (size_t)rs * a.h_in;
    switch (rs) {  // uniform over the wavefront
        case 8: gemv_expand_body<E, 1>(a, it, c0, c1, Bp, ho); break;
        case 16: gemv_expand_body<E, 2>(a, it, c0, c1, Bp, ho); break;
        case 32: gemv_expand_body<E, 4>(a, it, c0, c1, Bp, ho); break;
        case 64: gemv_expand_body<E, 8>(a, it, c0, c1, Bp, ho); break;
        case 128: gemv_expand_body<E, 16>(a, it, c0, c1, Bp, ho); break;
        default: gemv_expand_generic<E>(a, it, c0, c1, Bp, ho, vs); break;
    }
}

// ---------------------------------------------------------------------------------------
// kernels
// ---------------------------------------------------------------------------------------
template <typename E, int R>
__global__ __launch_bounds__(256) void gemv_shrink_kernel(ApplyArgs a, const GemvItem *__restrict__ items)
{
    constexpr int W = 4 / R;
    __shared__ float red[4][TB];
    const GemvItem it = items[blockIdx.x / W];
    gemv_shrink_block<E, R>(a, it, blockIdx.x % W, Handover{nullptr, 0, nullptr}, red);
}

template <typename E>
__global__ __launch_bounds__(64) void gemv_expand_kernel(ApplyArgs a, const GemvItem *__restrict__ items)
{
    __shared__ __attribute__((aligned(16))) float vs[TB][LORA_MAX_RANK];
    const GemvItem it = items[blockIdx.x];
    gemv_expand_wave<E>(a, it, blockIdx.y, Handover{nullptr, 0, nullptr}, vs);
}

// Fused: blocks [0, n_shrink_blocks) are shrink blocks, the rest hold four expand wavefronts
// each.  Blocks are dispatched in index order, so every shrink block is running or done by the
// time an expand wavefront starts to wait, and shrink blocks wait for nothing.
template <typename E, int R>
__global__ __launch_bounds__(256) void gemv_fused_kernel(ApplyArgs a, const GemvItem *__restrict__ gs,
                                                         const GemvItem *__restrict__ ge, int n_shrink_blocks, int n_ge,
                                                         int n_super, Handover ho)
{
    constexpr int W = 4 / R;
    __shared__ float red[4][TB];
    __shared__ __attribute__((aligned(16))) float vs[4][TB][LORA_MAX_RANK];
    if ((int)blockIdx.x < n_shrink_blocks) {
        const GemvItem it = gs[blockIdx.x / W];
        gemv_shrink_block<E, R>(a, it, blockIdx.x % W, ho, red);
    } else {
        const int w = threadIdx.x >> 6;
        const int unit = ((int)blockIdx.x - n_shrink_blocks) * 4 + w;
        const int item = unit / n_super;
        if (item >= n_ge) return;
        const GemvItem it = ge[item];
        gemv_expand_wave<E>(a, it, unit - item * n_super, ho, vs[w]);
    }
}

static int rows_split(int h_in)
{
    // one pass of a wavefront covers 4096 elements of a row; longer rows are split over 2 or 4
    // wavefronts so that a row still takes one pass
    return h_in <= 4096 ? 1 : (h_in <= 8192 ? 2 : 4);
}

hipError_t launch_gemv_shrink(int dtype, const ApplyArgs &a, const GemvItem *items, int n_items, hipStream_t st,
                              const KernelTimer *tm)
{
    if (n_items <= 0) return hipSuccess;
    const int w = rows_split(a.h_in);
    const dim3 grid(n_items * w), block(256);
    if (dtype == LORA_BF16) {
        if (w == 1) launch_k(tm, LORA_K_GEMV_SHRINK, gemv_shrink_kernel<__bf16, 4>, grid, block, st, a, items);
        else if (w == 2) launch_k(tm, LORA_K_GEMV_SHRINK, gemv_shrink_kernel<__bf16, 2>, grid, block, st, a, items);
        else launch_k(tm, LORA_K_GEMV_SHRINK, gemv_shrink_kernel<__bf16, 1>, grid, block, st, a, items);
    } else {
        if (w == 1) launch_k(tm, LORA_K_GEMV_SHRINK, gemv_shrink_kernel<float, 4>, grid, block, st, a, items);
        else if (w == 2) launch_k(tm, LORA_K_GEMV_SHRINK, gemv_shrink_kernel<float, 2>, grid, block, st, a, items);
        else launch_k(tm, LORA_K_GEMV_SHRINK, gemv_shrink_kernel<float, 1>, grid, block, st, a, items);
    }
    return hipGetLastError();
}

hipError_t launch_gemv_expand(int dtype, const ApplyArgs &a, const GemvItem *items, int n_items, hipStream_t st,
                              const KernelTimer *tm)
{
    if (n_items <= 0) return hipSuccess;
    const dim3 grid(n_items, (a.h_out + 1023) / 1024);
    if (dtype == LORA_BF16) launch_k(tm, LORA_K_GEMV_EXPAND, gemv_expand_kernel<__bf16>, grid, dim3(64), st, a, items);
    else launch_k(tm, LORA_K_GEMV_EXPAND, gemv_expand_kernel<float>, grid, dim3(64), st, a, items);
    return hipGetLastError();
}

hipError_t launch_gemv_fused(int dtype, const ApplyArgs &a, const GemvItem *gs, int n_gs, const GemvItem *ge, int n_ge,
                             int32_t *counters, int32_t epoch, int32_t *fault, hipStream_t st, const KernelTimer *tm)
{
    if (n_gs <= 0 || n_ge <= 0) return hipSuccess;
    const int w = rows_split(a.h_in);
    const int n_super = (a.h_out + 1023) / 1024;
    const int n_shrink_blocks = n_gs * w;
    const int n_expand_blocks = (n_ge * n_super + 3) / 4;
    const dim3 grid(n_shrink_blocks + n_expand_blocks), block(256);
    const Handover ho{counters, epoch, fault};
#define LORA_FUSED(E, R) \
    launch_k(tm, LORA_K_GEMV_FUSED, gemv_fused_kernel<E, R>, grid, block, st, a, gs, ge, n_shrink_blocks, n_ge, n_super, ho)
    if (dtype == LORA_BF16) {
        if (w == 1) LORA_FUSED(__bf16, 4);
        else if (w == 2) LORA_FUSED(__bf16, 2);
        else LORA_FUSED(__bf16, 1);
    } else {
        if (w == 1) LORA_FUSED(float, 4);
        else if (w == 2) LORA_FUSED(float, 2);
        else LORA_FUSED(float, 1);
    }
#undef LORA_FUSED
    return hipGetLastError();
}

}  // namespace lora
