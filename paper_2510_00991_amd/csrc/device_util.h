// Device-side helpers shared by the copy and MoE kernels: the 16-byte vector type
// and the load / store cache policies.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace vccl {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Access policy POL: 0 plain; 1 non-temporal loads and stores; 2 non-temporal
// loads, stores marked device scope (sc1), which measured 1.5 % faster than the
// non-temporal store on this chip.  The device-scope store is issued as a raw
// buffer store (the builtin that exposes the cache-policy bits) through a
// descriptor built on the wave-uniform tile base; lane offsets stay below 2 GiB.
template <int POL>
__device__ __forceinline__ u32x4 ld16(const u32x4 *p) {
    if (POL >= 1) return __builtin_nontemporal_load(p);
    return *p;
}
template <int POL>
struct TileDst {
    u32x4 *base;
    __amdgpu_buffer_rsrc_t rsrc;
    // `base` must be the same in every lane of the wavefront.
    __device__ __forceinline__ explicit TileDst(u32x4 *b) : base(b) {
        if (POL == 2)
            rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)b, 0, 0x7fffffff, 0x00020000 /* raw dwords */);
    }
    __device__ __forceinline__ void store(uint32_t idx, u32x4 v) const {
        if (POL == 2) __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, idx * 16u, 0, 16 /* sc1 */);
        else if (POL == 1) __builtin_nontemporal_store(v, base + idx);
        else base[idx] = v;
    }
};

// Division of a block index by a launch-time constant without a division: for
// 0 <= x < 2^31 and 1 <= d < 2^31, floor(x / d) = (x * m) >> s with l = ceil(log2 d),
// s = 31 + l, m = ceil(2^s / d) (m < 2^33, so the product fits 64 bits).
struct FastDiv {
    uint64_t m;
    uint32_t s;
    uint32_t d;
    FastDiv() = default;
    explicit FastDiv(uint32_t divisor) : d(divisor) {
        uint32_t l = 0;
        while ((1ull << l) < divisor) ++l;
        s = 31 + l;
        m = ((1ull << s) + divisor - 1) / divisor;
    }
    __device__ __forceinline__ uint32_t div(uint32_t x) const { return (uint32_t)(((uint64_t)x * m) >> s); }
};

}  // namespace vccl
