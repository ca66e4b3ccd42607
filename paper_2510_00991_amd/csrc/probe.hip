// Co-run probe: a compute-bound kernel with no memory traffic, launched as one
// wave of workgroups over all compute units - the shape of the GEMM whose tail
// the paper sees stretched by co-resident communication warps (Appendix E).
// Its run time alone versus beside a transfer is the co-run slowdown.
#include "common.h"
#include "device_util.h"

namespace vccl {

// CLOCKS: every workgroup also reports how long it ran on two of the chip's counters -
// the shader clock (which power management raises and lowers) and the constant-rate
// real-time counter - so that a longer run time can be told apart: more cycles means the
// workgroup was held up inside its compute unit, the same cycles at a lower clock means
// the chip slowed its shaders down.
template <bool CLOCKS>
__global__ void fma_probe_kernel(float *out, uint64_t iters, uint64_t *clocks) {
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    uint64_t c0 = 0, r0 = 0;
    if (CLOCKS) {
        c0 = clock64();
        r0 = wall_clock64();
    }
    // eight independent dependency chains per lane keep the FMA pipe full
    float a0 = 1.0f + gid * 1e-7f, a1 = a0 + 0.125f, a2 = a0 + 0.25f, a3 = a0 + 0.375f;
    float a4 = a0 + 0.5f, a5 = a0 + 0.625f, a6 = a0 + 0.75f, a7 = a0 + 0.875f;
    const float m = 0.99999994f, c = 1.0e-6f;
    for (uint64_t i = 0; i < iters; ++i) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            a0 = __builtin_fmaf(a0, m, c);
            a1 = __builtin_fmaf(a1, m, c);
            a2 = __builtin_fmaf(a2, m, c);
            a3 = __builtin_fmaf(a3, m, c);
            a4 = __builtin_fmaf(a4, m, c);
            a5 = __builtin_fmaf(a5, m, c);
            a6 = __builtin_fmaf(a6, m, c);
            a7 = __builtin_fmaf(a7, m, c);
        }
    }
    out[gid] = ((a0 + a1) + (a2 + a3)) + ((a4 + a5) + (a6 + a7));
    if (CLOCKS) {
        const uint64_t c1 = clock64(), r1 = wall_clock64();
        if (threadIdx.x == 0) {
            clocks[2 * (size_t)blockIdx.x] = c1 - c0;
            clocks[2 * (size_t)blockIdx.x + 1] = r1 - r0;
        }
    }
}

int launch_fma_probe(float *out, uint64_t *clocks, uint32_t workgroups, uint32_t threads, uint64_t iters,
                     hipStream_t stream) {
    if (clocks) fma_probe_kernel<true><<<dim3(workgroups), dim3(threads), 0, stream>>>(out, iters, clocks);
    else fma_probe_kernel<false><<<dim3(workgroups), dim3(threads), 0, stream>>>(out, iters, nullptr);
    VCCL_HIP(hipGetLastError());
    return VCCL_OK;
}

// ---- HBM ceiling probes: plain streaming kernels with the launch shapes of the copy
// paths, so that what the chip gives for read-only, write-only, copy and
// scattered-row-write traffic can be measured beside them.  One workgroup of T lanes
// handles V consecutive 16-byte vectors per lane (a contiguous run of T*V*16 bytes).
template <int T, int V>
__global__ __launch_bounds__(T) void hbm_read_kernel(const u32x4 *src, uint64_t nvec, u32x4 *sink) {
    const uint64_t base = (uint64_t)blockIdx.x * (T * V);
    u32x4 acc = {0, 0, 0, 0};
#pragma unroll
    for (int u = 0; u < V; ++u) {
        const uint64_t i = base + (uint64_t)u * T + threadIdx.x;
        if (i < nvec) acc ^= __builtin_nontemporal_load(src + i);
    }
    // never true for the probe's input, but the compiler cannot know: the loads stay
    if (acc.x == 0x9e3779b9u && acc.y == 0x7f4a7c15u && acc.z == 0xf39cc060u && acc.w == 0x5cedc834u) sink[0] = acc;
}

template <int T, int V>
__global__ __launch_bounds__(T) void hbm_write_kernel(u32x4 *dst, uint64_t nvec) {
    const uint64_t base = (uint64_t)blockIdx.x * (T * V);
    const TileDst<2> d(dst + base);
    const u32x4 v = {blockIdx.x, threadIdx.x, 0x5a5a5a5au, 0xa5a5a5a5u};
#pragma unroll
    for (int u = 0; u < V; ++u) {
        const uint32_t i = (uint32_t)u * T + threadIdx.x;
        if (base + i < nvec) d.store(i, v);
    }
}

template <int T, int V>
__global__ __launch_bounds__(T) void hbm_copy_kernel(const u32x4 *src, u32x4 *dst, uint64_t nvec) {
    const uint64_t base = (uint64_t)blockIdx.x * (T * V);
    const TileDst<2> d(dst + base);
    u32x4 r[V];
#pragma unroll
    for (int u = 0; u < V; ++u) {
        const uint64_t i = base + (uint64_t)u * T + threadIdx.x;
        if (i < nvec) r[u] = __builtin_nontemporal_load(src + i);
    }
#pragma unroll
    for (int u = 0; u < V; ++u) {
        const uint32_t i = (uint32_t)u * T + threadIdx.x;
        if (base + i < nvec) d.store(i, r[u]);
    }
}

// Rows of row_vecs vectors written whole, row i of the launch going to row
// row_index[i] of dst (i itself if row_index is null); one workgroup per run of T*V
// vectors of a row.
template <int T, int V>
__global__ __launch_bounds__(T) void hbm_write_rows_kernel(u32x4 *dst, const uint32_t *row_index, uint32_t row_vecs,
                                                           uint32_t runs_per_row, uint64_t n_rows) {
    const uint64_t i = blockIdx.x / runs_per_row;
    const uint32_t run = blockIdx.x - (uint32_t)i * runs_per_row;
    if (i >= n_rows) return;
    const uint64_t row = row_index ? row_index[i] : i;
    const uint32_t v0 = run * (T * V);
    const TileDst<2> d(dst + row * row_vecs + v0);
    const u32x4 v = {(uint32_t)i, threadIdx.x, 0x5a5a5a5au, 0xa5a5a5a5u};
#pragma unroll
    for (int u = 0; u < V; ++u) {
        const uint32_t k = (uint32_t)u * T + threadIdx.x;
        if (v0 + k < row_vecs) d.store(k, v);
    }
}

template <int T, int V>
static int launch_hbm_shape(int kind, const void *src, void *dst, uint64_t bytes, const uint32_t *row_index,
                            uint64_t n_rows, uint64_t row_bytes, hipStream_t stream) {
    const uint64_t nvec = bytes >> 4;
    const uint64_t per_wg = (uint64_t)T * V;
    if (kind == 3) {
        const uint32_t row_vecs = (uint32_t)(row_bytes >> 4);
        const uint32_t runs = (uint32_t)((row_vecs + per_wg - 1) / per_wg);
        const uint64_t grid = n_rows * runs;
        if (grid == 0 || grid > 0x7fffffffull) return fail(VCCL_ERR_ARG, "rows x runs = %llu does not fit a launch", (unsigned long long)grid);
        hbm_write_rows_kernel<T, V><<<dim3((uint32_t)grid), dim3(T), 0, stream>>>((u32x4 *)dst, row_index, row_vecs, runs, n_rows);
    } else {
        const uint64_t grid = (nvec + per_wg - 1) / per_wg;
        if (grid == 0 || grid > 0x7fffffffull) return fail(VCCL_ERR_ARG, "%llu bytes do not fit a launch of this shape", (unsigned long long)bytes);
        if (kind == 0) hbm_read_kernel<T, V><<<dim3((uint32_t)grid), dim3(T), 0, stream>>>((const u32x4 *)src, nvec, (u32x4 *)dst);
        else if (kind == 1) hbm_write_kernel<T, V><<<dim3((uint32_t)grid), dim3(T), 0, stream>>>((u32x4 *)dst, nvec);
        else hbm_copy_kernel<T, V><<<dim3((uint32_t)grid), dim3(T), 0, stream>>>((const u32x4 *)src, (u32x4 *)dst, nvec);
    }
    VCCL_HIP(hipGetLastError());
    return VCCL_OK;
}

int launch_hbm_probe(int kind, const void *src, void *dst, uint64_t bytes, int threads, int vecs,
                     const uint32_t *row_index, uint64_t n_rows, uint64_t row_bytes, hipStream_t stream) {
#define VCCL_SHAPE(T, V) \
    if (threads == T && vecs == V) return launch_hbm_shape<T, V>(kind, src, dst, bytes, row_index, n_rows, row_bytes, stream)
    VCCL_SHAPE(64, 1);
    VCCL_SHAPE(64, 2);
    VCCL_SHAPE(64, 4);
    VCCL_SHAPE(64, 16);
    VCCL_SHAPE(256, 1);
    VCCL_SHAPE(256, 4);
    VCCL_SHAPE(448, 2);
#undef VCCL_SHAPE
    return fail(VCCL_ERR_ARG, "shape %d lanes x %d vectors is not one of 64x1, 64x2, 64x4, 64x16, 256x1, 256x4, 448x2",
                threads, vecs);
}

}  // namespace vccl
