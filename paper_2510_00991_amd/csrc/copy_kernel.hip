// Compute-unit copy path: one descriptor-driven kernel moves every segment of a
// SendRecv / AlltoAll(v) call.  This is the kind of P2P copy kernel that occupies
// compute units for the whole transfer (paper Section 2.2, intra-node pattern;
// Appendix A), written here for CDNA4: 64-lane wavefronts, each lane moving 16
// bytes per instruction, a wavefront's access covering 1 KiB of contiguous HBM.
//
// Work decomposition: a segment is split into a bytewise head (until the
// destination is 16-byte aligned), a body of 16-byte vectors cut into tiles of
// U*256 vectors, and a bytewise tail.  Tiles of all segments are numbered
// consecutively; a persistent grid strides over them.  When source and
// destination of a body disagree modulo 16 the tile goes through LDS: aligned
// 16-byte global loads, a byte funnel shift in registers, aligned 16-byte stores.
#include "common.h"

namespace vccl {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct CopyArgs {
    const Seg *table;       // device descriptor table, or nullptr: use inl[]
    uint32_t nseg;
    uint32_t total_tiles;
    uint32_t uniform_tiles; // > 0: every segment owns exactly this many tiles
    uint32_t xcd_map;       // 1: give each XCD one contiguous eighth of the tiles
    Seg inl[kInlineSegs];
};

constexpr int kLdsVecs = 1024;  // vectors staged per LDS round of the realign path

template <bool NT>
__device__ __forceinline__ u32x4 ld16(const u32x4 *p) {
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}
template <bool NT>
__device__ __forceinline__ void st16(u32x4 *p, u32x4 v) {
    if (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// Last segment whose first tile is <= tile; the 64 lanes probe 64 evenly spaced
// descriptors per round, so 4096 segments need two rounds.  Result is wave-uniform.
__device__ __forceinline__ uint32_t find_segment(const Seg *segs, uint32_t nseg, uint32_t tile,
                                                 uint32_t lane) {
    uint32_t lo = 0, n = nseg;
    while (n > 1) {
        const uint32_t step = (n + 63u) >> 6;
        const uint32_t off = lane * step;
        const bool le = off < n && segs[lo + off].tile_begin <= tile;
        const uint32_t c = (uint32_t)__popcll(__ballot(le));
        const uint32_t adv = (c - 1u) * step;
        n = min(step, n - adv);
        lo += adv;
    }
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)lo);
}

__device__ __forceinline__ uint32_t funnel(uint32_t lo, uint32_t hi, uint32_t byte_shift) {
    return (uint32_t)((((uint64_t)hi << 32) | lo) >> (8u * byte_shift));
}

template <int U, bool NT>
__global__ __launch_bounds__(kCopyThreads) void copy_segments_kernel(CopyArgs by_value) {
    (void)by_value;
    // The argument block is read in place (dynamic indexing of a by-value
    // aggregate could otherwise be spilled to private memory).
    const CopyArgs *a =
        reinterpret_cast<const CopyArgs *>((const void *)__builtin_amdgcn_kernarg_segment_ptr());
    const Seg *segs = a->table ? a->table : a->inl;
    const uint32_t nseg = a->nseg;
    const uint32_t total = a->total_tiles;
    const uint32_t uniform = a->uniform_tiles;
    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63u;
    constexpr uint32_t kTileVecs = (uint32_t)U * kCopyThreads;

    __shared__ u32x4 stage[kLdsVecs + 1];

    uint32_t t, t_end, t_step;
    if (a->xcd_map) {
        // Consecutive workgroup ids land on consecutive XCDs; keep each XCD inside
        // its own contiguous range of tiles.
        const uint32_t xcd = blockIdx.x & 7u;
        const uint32_t per = (total + 7u) >> 3;
        t = xcd * per + (blockIdx.x >> 3);
        t_end = min(total, (xcd + 1u) * per);
        t_step = gridDim.x >> 3;
    } else {
        t = blockIdx.x;
        t_end = total;
        t_step = gridDim.x;
    }

    for (; t < t_end; t += t_step) {
        uint32_t si, k;
        if (uniform) {
            si = t / uniform;
            k = t - si * uniform;
        } else {
            si = find_segment(segs, nseg, t, lane);
            k = t - segs[si].tile_begin;
        }
        const uint8_t *src = segs[si].src;
        uint8_t *dst = segs[si].dst;
        const uint64_t bytes = segs[si].bytes;
        const uint32_t head = segs[si].head;
        const uint64_t body = bytes - head;
        const uint64_t nv = body >> 4;
        if (k == 0) {
            const uint32_t tail = (uint32_t)(body & 15u);
            if (tid < head) {
                dst[tid] = src[tid];
            } else if (tid >= 64u && tid < 64u + tail) {
                const uint64_t o = head + (nv << 4) + (tid - 64u);
                dst[o] = src[o];
            }
        }
        const uint64_t v0 = (uint64_t)k * kTileVecs;
        if (v0 >= nv) continue;
        const uint32_t cnt = (uint32_t)min((uint64_t)kTileVecs, nv - v0);
        const uint8_t *sb = src + head + (v0 << 4);
        u32x4 *d = reinterpret_cast<u32x4 *>(dst + head + (v0 << 4));
        const uint32_t mis = (uint32_t)(reinterpret_cast<uintptr_t>(sb) & 15u);
        if (mis == 0) {
            const u32x4 *s = reinterpret_cast<const u32x4 *>(sb);
            if (cnt == kTileVecs) {
                u32x4 r[U];
#pragma unroll
                for (int u = 0; u < U; ++u) r[u] = ld16<NT>(s + u * kCopyThreads + tid);
#pragma unroll
                for (int u = 0; u < U; ++u) st16<NT>(d + u * kCopyThreads + tid, r[u]);
            } else {
                for (uint32_t i = tid; i < cnt; i += kCopyThreads) st16<NT>(d + i, ld16<NT>(s + i));
            }
        } else {
            // Every aligned word read below holds at least one byte of the segment
            // (mis > 0), so it lies on a page the segment itself touches.
            const u32x4 *sa = reinterpret_cast<const u32x4 *>(sb - mis);
            const uint32_t q = mis >> 2, sh = mis & 3u;
            for (uint32_t c0 = 0; c0 < cnt; c0 += kLdsVecs) {
                const uint32_t m = min((uint32_t)kLdsVecs, cnt - c0);
                __syncthreads();
                for (uint32_t i = tid; i < m; i += kCopyThreads) stage[i] = ld16<NT>(sa + c0 + i);
                if (tid == 0) stage[m] = ld16<NT>(sa + c0 + m);
                __syncthreads();
                for (uint32_t i = tid; i < m; i += kCopyThreads) {
                    const u32x4 lo = stage[i], hi = stage[i + 1];
                    const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                    u32x4 o;
                    switch (q) {  // wave-uniform
                        case 0: o = u32x4{funnel(w[0], w[1], sh), funnel(w[1], w[2], sh),
                                          funnel(w[2], w[3], sh), funnel(w[3], w[4], sh)}; break;
                        case 1: o = u32x4{funnel(w[1], w[2], sh), funnel(w[2], w[3], sh),
                                          funnel(w[3], w[4], sh), funnel(w[4], w[5], sh)}; break;
                        case 2: o = u32x4{funnel(w[2], w[3], sh), funnel(w[3], w[4], sh),
                                          funnel(w[4], w[5], sh), funnel(w[5], w[6], sh)}; break;
                        default: o = u32x4{funnel(w[3], w[4], sh), funnel(w[4], w[5], sh),
                                           funnel(w[5], w[6], sh), funnel(w[6], w[7], sh)}; break;
                    }
                    st16<NT>(d + c0 + i, o);
                }
            }
        }
    }
}

int plan_tiles(CopyPlan &plan, int unroll) {
    const uint64_t tile_vecs = (uint64_t)unroll * kCopyThreads;
    uint64_t tiles = 0;
    uint64_t first = 0;
    bool uniform = true;
    plan.bytes = 0;
    for (size_t i = 0; i < plan.segs.size(); ++i) {
        Seg &s = plan.segs[i];
        const uint64_t to_align = (16u - (reinterpret_cast<uintptr_t>(s.dst) & 15u)) & 15u;
        s.head = (uint32_t)(s.bytes < to_align ? s.bytes : to_align);
        const uint64_t nv = (s.bytes - s.head) >> 4;
        uint64_t nt = (nv + tile_vecs - 1) / tile_vecs;
        if (nt == 0) nt = 1;
        if (i == 0) first = nt;
        else if (nt != first) uniform = false;
        if (tiles + nt > 0x7fffffffull)
            return fail(VCCL_ERR_UNSUPPORTED, "exchange needs more than 2^31 copy tiles");
        s.tile_begin = (uint32_t)tiles;
        tiles += nt;
        plan.bytes += s.bytes;
    }
    plan.total_tiles = (uint32_t)tiles;
    plan.uniform_tiles = (uniform && !plan.segs.empty()) ? (uint32_t)first : 0;
    return VCCL_OK;
}

template <int U>
static void launch_variant(bool nt, dim3 grid, hipStream_t stream, const CopyArgs &args) {
    if (nt) copy_segments_kernel<U, true><<<grid, dim3(kCopyThreads), 0, stream>>>(args);
    else copy_segments_kernel<U, false><<<grid, dim3(kCopyThreads), 0, stream>>>(args);
}

int launch_copy(const CopyPlan &plan, const Options &opt, int cu_count, DescRing &ring,
                hipStream_t stream) {
    if (plan.segs.empty() || plan.total_tiles == 0) return VCCL_OK;
    CopyArgs args;
    args.table = nullptr;
    args.nseg = (uint32_t)plan.segs.size();
    args.total_tiles = plan.total_tiles;
    args.uniform_tiles = plan.uniform_tiles;
    DescSlot *slot = nullptr;
    if (plan.segs.size() <= (size_t)kInlineSegs) {
        for (size_t i = 0; i < plan.segs.size(); ++i) args.inl[i] = plan.segs[i];
    } else {
        if (plan.segs.size() > ring.capacity)
            return fail(VCCL_ERR_ARG, "%zu segments exceed the descriptor ring capacity %zu",
                        plan.segs.size(), ring.capacity);
        int rv = ring.acquire(&slot);
        if (rv) return rv;
        for (size_t i = 0; i < plan.segs.size(); ++i) slot->host[i] = plan.segs[i];
        VCCL_HIP(hipMemcpyAsync(slot->dev, slot->host, plan.segs.size() * sizeof(Seg),
                                hipMemcpyHostToDevice, stream));
        args.table = slot->dev;
    }
    uint64_t g = (uint64_t)cu_count * (uint64_t)opt.cu_wg_per_cu;
    if (opt.cu_max_wg > 0 && g > (uint64_t)opt.cu_max_wg) g = (uint64_t)opt.cu_max_wg;
    if (g > plan.total_tiles) g = plan.total_tiles;
    if (g < 1) g = 1;
    args.xcd_map = (opt.cu_xcd_map && (g % 8 == 0) && plan.total_tiles >= 8 * g) ? 1u : 0u;
    const dim3 grid((uint32_t)g);
    const bool nt = opt.cu_nontemporal != 0;
    switch (opt.cu_unroll) {
        case 1: launch_variant<1>(nt, grid, stream, args); break;
        case 2: launch_variant<2>(nt, grid, stream, args); break;
        case 4: launch_variant<4>(nt, grid, stream, args); break;
        case 8: launch_variant<8>(nt, grid, stream, args); break;
        case 16: launch_variant<16>(nt, grid, stream, args); break;
        default: return fail(VCCL_ERR_ARG, "cu_unroll %d is not one of 1,2,4,8,16", opt.cu_unroll);
    }
    VCCL_HIP(hipGetLastError());
    if (slot) VCCL_HIP(hipEventRecord(slot->done, stream));
    return VCCL_OK;
}

}  // namespace vccl
