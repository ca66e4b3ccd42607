// Co-run probe: a compute-bound kernel with no memory traffic, launched as one
// wave of workgroups over all compute units - the shape of the GEMM whose tail
// the paper sees stretched by co-resident communication warps (Appendix E).
// Its run time alone versus beside a transfer is the co-run slowdown.
#include "common.h"

namespace vccl {

__global__ void fma_probe_kernel(float *out, uint64_t iters) {
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
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
}

int launch_fma_probe(float *out, uint32_t workgroups, uint32_t threads, uint64_t iters,
                     hipStream_t stream) {
    fma_probe_kernel<<<dim3(workgroups), dim3(threads), 0, stream>>>(out, iters);
    VCCL_HIP(hipGetLastError());
    return VCCL_OK;
}

}  // namespace vccl
