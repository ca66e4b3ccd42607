// Compute-unit copy path: one descriptor-driven kernel moves every segment of a
// SendRecv / AlltoAll(v) call.  This is the kind of P2P copy kernel that occupies
// compute units for the whole transfer (paper Section 2.2, intra-node pattern;
// Appendix A), written here for CDNA4: 64-lane wavefronts, each lane moving 16
// bytes per instruction, a wavefront's access covering 1 KiB of contiguous HBM.
//
// Work decomposition: a segment is split into a bytewise head (until the
// destination is 16-byte aligned), a body of 16-byte vectors cut into tiles of
// U*T vectors (T lanes per workgroup, 64 by default) at destination addresses
// that are multiples of the tile size, and a bytewise tail.  The grid is
// two-dimensional: blockIdx.y
// names the descriptor, blockIdx.x the tile inside it, so a workgroup finds its
// work with one scalar load and no search.  The host planner cuts long segments
// into pieces so that all descriptors have about the same number of tiles.
// One small tile per workgroup keeps the set of addresses in flight at any
// moment inside a few MiB that sweep forward through the buffers, which is what
// HBM rewards; a capped grid (for the co-run study) strides over tiles instead.
// When source and destination of a body disagree modulo 16 each lane loads the
// two aligned words that cover its vector and funnel-shifts them in registers:
// aligned 16-byte loads, aligned 16-byte stores.
#include "common.h"
#include "device_util.h"

namespace vccl {


struct CopyArgs {
    const Seg *table;       // device descriptor table (unused by the inline variant)
    uint32_t nseg;
    uint32_t pad;
    Seg inl[kInlineSegs];
};

__device__ __forceinline__ uint32_t funnel(uint32_t lo, uint32_t hi, uint32_t byte_shift) {
    return (uint32_t)((((uint64_t)hi << 32) | lo) >> (8u * byte_shift));
}

// Output vector made of bytes [mis, mis + 16) of the 32 bytes lo:hi (0 < mis < 16).
__device__ __forceinline__ u32x4 realign(u32x4 lo, u32x4 hi, uint32_t q, uint32_t sh) {
    const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    switch (q) {  // wave-uniform
        case 0: return u32x4{funnel(w[0], w[1], sh), funnel(w[1], w[2], sh), funnel(w[2], w[3], sh),
                             funnel(w[3], w[4], sh)};
        case 1: return u32x4{funnel(w[1], w[2], sh), funnel(w[2], w[3], sh), funnel(w[3], w[4], sh),
                             funnel(w[4], w[5], sh)};
        case 2: return u32x4{funnel(w[2], w[3], sh), funnel(w[3], w[4], sh), funnel(w[4], w[5], sh),
                             funnel(w[5], w[6], sh)};
        default: return u32x4{funnel(w[3], w[4], sh), funnel(w[4], w[5], sh), funnel(w[5], w[6], sh),
                              funnel(w[6], w[7], sh)};
    }
}

// General kernel: any byte alignment, any grid (workgroups stride over descriptors
// and tiles when the grid is capped).  A segment is head bytes (until the
// destination is 16-byte aligned), body vectors, tail bytes.  When the body's
// source is not 16-byte aligned each lane loads the two aligned words that cover
// its output vector (the second is its neighbour's first and comes from cache) and
// funnel-shifts them in registers: aligned loads, aligned stores, no LDS, no barrier.
template <int U, int NT, bool INLINE, int T>
__global__ __launch_bounds__(T) void copy_segments_kernel(CopyArgs by_value) {
    (void)by_value;
    // The argument block is read in place (dynamic indexing of a by-value
    // aggregate could otherwise be spilled to private memory).
    const CopyArgs *a =
        reinterpret_cast<const CopyArgs *>((const void *)__builtin_amdgcn_kernarg_segment_ptr());
    const Seg *segs = INLINE ? a->inl : a->table;
    const uint32_t nseg = a->nseg;
    const uint32_t tid = threadIdx.x;
    constexpr uint32_t kTileVecs = (uint32_t)U * T;

    for (uint32_t si = blockIdx.y; si < nseg; si += gridDim.y) {
        const uint8_t *src = segs[si].src;
        uint8_t *dst = segs[si].dst;
        const uint64_t bytes = segs[si].bytes;
        const uint32_t head = segs[si].head;
        const uint64_t body = bytes - head;
        const uint64_t nv = body >> 4;
        if (blockIdx.x == 0) {
            const uint32_t tail = (uint32_t)(body & 15u);
            if (tid < head) {
                dst[tid] = src[tid];
            } else if (tid >= 16u && tid < 16u + tail) {
                const uint64_t o = head + (nv << 4) + (tid - 16u);
                dst[o] = src[o];
            }
        }
        // Tiles are cut at destination addresses that are multiples of the tile size
        // (`lead` vectors precede the segment's body inside its first tile), so a
        // wavefront's stores cover whole cache lines whatever the buffer offset.
        const uint32_t lead = segs[si].lead;
        const uint64_t ntiles = (nv + lead + kTileVecs - 1) / kTileVecs;
        for (uint64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
            const uint64_t end = (tile + 1) * kTileVecs - lead;   // >= 1
            const uint64_t v0 = tile ? tile * kTileVecs - lead : 0;
            const uint32_t cnt = (uint32_t)(min(end, nv) - v0);
            const uint8_t *sb = src + head + (v0 << 4);
            const TileDst<NT> d(reinterpret_cast<u32x4 *>(dst + head + (v0 << 4)));
            const uint32_t mis = (uint32_t)(reinterpret_cast<uintptr_t>(sb) & 15u);
            if (mis == 0) {
                const u32x4 *s = reinterpret_cast<const u32x4 *>(sb);
                if (cnt == kTileVecs) {
                    u32x4 r[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) r[u] = ld16<NT>(s + u * T + tid);
#pragma unroll
                    for (int u = 0; u < U; ++u) d.store(u * T + tid, r[u]);
                } else {
                    for (uint32_t i = tid; i < cnt; i += T) d.store(i, ld16<NT>(s + i));
                }
            } else {
                // Output vector i is bytes [mis, mis + 16) of aligned words i and i + 1.
                // Both hold at least one byte of the segment (0 < mis < 16), so they lie
                // on pages the segment itself touches.
                const u32x4 *sa = reinterpret_cast<const u32x4 *>(sb - mis);
                const uint32_t q = mis >> 2, sh = mis & 3u;
                if (cnt == kTileVecs) {
                    u32x4 lo[U], hi[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        lo[u] = ld16<NT>(sa + u * T + tid);
                        hi[u] = ld16<0>(sa + u * T + tid + 1);
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) d.store(u * T + tid, realign(lo[u], hi[u], q, sh));
                } else {
                    for (uint32_t i = tid; i < cnt; i += T)
                        d.store(i, realign(ld16<NT>(sa + i), ld16<0>(sa + i + 1), q, sh));
                }
            }
        }
    }
}

// Fast path for the common case in which every descriptor starts at 16-byte aligned
// addresses on both sides and is a whole number of vectors long (all five
// workload configurations): no head, tail, realignment or loop - one scalar
// descriptor load, U vector loads, U vector stores.  Needs the full grid.
template <int U, int NT, bool INLINE, int T>
__global__ __launch_bounds__(T) void copy_aligned_kernel(CopyArgs by_value) {
    (void)by_value;
    const CopyArgs *a =
        reinterpret_cast<const CopyArgs *>((const void *)__builtin_amdgcn_kernarg_segment_ptr());
    // the whole 32-byte descriptor in one scalar load, before any branch
    const Seg *sp = (INLINE ? a->inl : a->table) + blockIdx.y;
    const uint8_t *seg_src = sp->src;
    uint8_t *seg_dst = sp->dst;
    const uint64_t seg_bytes = sp->bytes;
    const uint32_t lead = sp->lead;
    // (an empty statement that needs both pointers in registers here: without it the
    // compiler moves their load behind the first branch and the wavefront waits twice)
    asm volatile("" ::"s"(seg_src), "s"(seg_dst));
    constexpr uint32_t kTileVecs = (uint32_t)U * T;
    // 32-bit vector counts (the planner gives this kernel no segment of 64 GiB or more):
    // the bounds tests stay on the scalar unit
    const uint32_t nv = (uint32_t)(seg_bytes >> 4);
    // tile 0 holds the `lead` vectors' worth of room before the segment, so that
    // every later tile starts on a destination address that is a multiple of the tile
    // (no 32-bit overflow: the grid has at most ceil((nv + lead) / tile) columns and
    // nv <= 0xffff0000, tiles are at most 4096 vectors)
    const uint32_t start = blockIdx.x * kTileVecs;
    const uint32_t v0 = blockIdx.x ? start - lead : 0;
    if (v0 >= nv) return;
    const uint32_t end = min(start + kTileVecs - lead, nv);
    const u32x4 *s = reinterpret_cast<const u32x4 *>(seg_src) + v0;
    const TileDst<NT> d(reinterpret_cast<u32x4 *>(seg_dst) + v0);
    const uint32_t tid = threadIdx.x;
    if (end - v0 == kTileVecs) {
        u32x4 r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) r[u] = ld16<NT>(s + u * T + tid);
#pragma unroll
        for (int u = 0; u < U; ++u) d.store(u * T + tid, r[u]);
    } else {
        const uint32_t cnt = end - v0;
        for (uint32_t i = tid; i < cnt; i += T) d.store(i, ld16<NT>(s + i));
    }
}

// Equal-block AlltoAll without a descriptor table: the P send and P receive
// pointers ride in the kernel arguments and a workgroup derives its segment from
// blockIdx.y - segment q = k*P + r moves block r of send[(r+k) mod P] to block
// (r+k) mod P of recv[r], the same rotated order the planner uses.  Nothing is
// uploaded, so a P = 64 exchange of small blocks costs one launch.
constexpr int kUniformRanks = 128;
struct UniformArgs {
    const uint8_t *send[kUniformRanks];
    uint8_t *recv[kUniformRanks];
    uint64_t vecs_per_block;   // bytes_per_peer / 16
    uint32_t P;
    uint32_t pad;
};

template <int U, int NT, int T>
__global__ __launch_bounds__(T) void copy_uniform_kernel(UniformArgs by_value) {
    (void)by_value;
    const UniformArgs *a =
        reinterpret_cast<const UniformArgs *>((const void *)__builtin_amdgcn_kernarg_segment_ptr());
    constexpr uint32_t kTileVecs = (uint32_t)U * T;
    const uint64_t nv = a->vecs_per_block;
    const uint32_t P = a->P;
    const uint32_t k = blockIdx.y / P, r = blockIdx.y - k * P;
    uint32_t s_rank = r + k;
    if (s_rank >= P) s_rank -= P;
    u32x4 *dseg = reinterpret_cast<u32x4 *>(a->recv[r]) + (uint64_t)s_rank * nv;
    // destination-aligned tiles, as in the descriptor kernels
    const uint32_t lead = (uint32_t)((reinterpret_cast<uintptr_t>(dseg) >> 4) & (kTileVecs - 1u));
    const uint64_t end = ((uint64_t)blockIdx.x + 1) * kTileVecs - lead;
    const uint64_t v0 = blockIdx.x ? (uint64_t)blockIdx.x * kTileVecs - lead : 0;
    if (v0 >= nv) return;
    const u32x4 *s = reinterpret_cast<const u32x4 *>(a->send[s_rank]) + (uint64_t)r * nv + v0;
    const TileDst<NT> d(dseg + v0);
    const uint32_t tid = threadIdx.x;
    if (end - v0 == kTileVecs && end <= nv) {
        u32x4 reg[U];
#pragma unroll
        for (int u = 0; u < U; ++u) reg[u] = ld16<NT>(s + u * T + tid);
#pragma unroll
        for (int u = 0; u < U; ++u) d.store(u * T + tid, reg[u]);
    } else {
        const uint32_t cnt = (uint32_t)(min(end, nv) - v0);
        for (uint32_t i = tid; i < cnt; i += T) d.store(i, ld16<NT>(s + i));
    }
}

bool uniform_alltoall_applies(void *const *sendbuf, void *const *recvbuf, uint64_t bytes_per_peer, int P,
                              const Options &opt) {
    if (!opt.cu_fast_path || opt.check || opt.cu_max_wg || opt.cu_wg_per_cu) return false;
    if (P > kUniformRanks || (uint64_t)P * P > 65535 || bytes_per_peer == 0 || (bytes_per_peer & 15u)) return false;
    const uint64_t tiles = ((bytes_per_peer >> 4) + (uint64_t)opt.cu_unroll * opt.cu_threads - 1) /
                           ((uint64_t)opt.cu_unroll * opt.cu_threads);
    if (tiles + 1 > 0x7fffffffull) return false;
    for (int i = 0; i < P; ++i)
        if (!sendbuf[i] || !recvbuf[i] ||
            ((reinterpret_cast<uintptr_t>(sendbuf[i]) | reinterpret_cast<uintptr_t>(recvbuf[i])) & 15u))
            return false;
    return true;
}

int launch_uniform_alltoall(void *const *sendbuf, void *const *recvbuf, uint64_t bytes_per_peer, int P,
                            const Options &opt, hipStream_t stream) {
    UniformArgs a;
    for (int i = 0; i < P; ++i) {
        a.send[i] = static_cast<const uint8_t *>(sendbuf[i]);
        a.recv[i] = static_cast<uint8_t *>(recvbuf[i]);
    }
    a.vecs_per_block = bytes_per_peer >> 4;
    a.P = (uint32_t)P;
    a.pad = 0;
    const uint64_t tile_vecs = (uint64_t)opt.cu_unroll * opt.cu_threads;   // a power of two
    // destination-aligned tiles: the longest lead over all blocks sizes the grid
    uint64_t max_lead = 0;
    for (int r = 0; r < P && max_lead + 1 < tile_vecs; ++r)
        for (int sr = 0; sr < P; ++sr) {
            const uint64_t lead =
                ((reinterpret_cast<uintptr_t>(recvbuf[r]) >> 4) + (uint64_t)sr * a.vecs_per_block) & (tile_vecs - 1);
            if (lead > max_lead) max_lead = lead;
        }
    const dim3 grid((uint32_t)((a.vecs_per_block + max_lead + tile_vecs - 1) / tile_vecs), (uint32_t)(P * P));
    const dim3 block((uint32_t)opt.cu_threads);
#define VCCL_UNI_T(U, POL)                                                                           \
    if (opt.cu_threads == 64) copy_uniform_kernel<U, POL, 64><<<grid, block, 0, stream>>>(a);        \
    else if (opt.cu_threads == 128) copy_uniform_kernel<U, POL, 128><<<grid, block, 0, stream>>>(a); \
    else copy_uniform_kernel<U, POL, 256><<<grid, block, 0, stream>>>(a)
#define VCCL_UNI(U)                                                                              \
    if (opt.cu_nontemporal == 2) { VCCL_UNI_T(U, 2); }                                           \
    else if (opt.cu_nontemporal == 1) { VCCL_UNI_T(U, 1); }                                      \
    else { VCCL_UNI_T(U, 0); }
    switch (opt.cu_unroll) {
        case 1: VCCL_UNI(1); break;
        case 2: VCCL_UNI(2); break;
        case 4: VCCL_UNI(4); break;
        case 8: VCCL_UNI(8); break;
        case 16: VCCL_UNI(16); break;
        default: return fail(VCCL_ERR_ARG, "cu_unroll %d is not one of 1,2,4,8,16", opt.cu_unroll);
    }
#undef VCCL_UNI
#undef VCCL_UNI_T
    VCCL_HIP(hipGetLastError());
    return VCCL_OK;
}

// Head bytes of a segment: what precedes the first 16-byte aligned destination address.
static inline uint32_t head_of(const uint8_t *dst, uint64_t bytes) {
    const uint64_t to_align = (16u - (reinterpret_cast<uintptr_t>(dst) & 15u)) & 15u;
    return (uint32_t)(bytes < to_align ? bytes : to_align);
}

int plan_tiles(CopyPlan &plan, int unroll, int threads, bool allow_fast) {
    plan.all_aligned = !plan.segs.empty();
    for (const Seg &s : plan.segs)
        if (((reinterpret_cast<uintptr_t>(s.src) | reinterpret_cast<uintptr_t>(s.dst) | s.bytes) & 15u) != 0) {
            plan.all_aligned = false;
            break;
        }
    // Cutting (below) adds at most 8192 pieces; the all-aligned kernel needs one
    // grid row per descriptor, and a grid has at most 65535 rows.
    plan.fast = plan.all_aligned && allow_fast && plan.segs.size() <= 65535u - 8192u;
    for (const Seg &s : plan.segs)   // the all-aligned kernel counts vectors in 32 bits
        if ((s.bytes >> 4) > 0xffff0000ull) plan.fast = false;
    plan.threads = threads;
    const uint64_t tile_vecs = (uint64_t)unroll * plan.threads;
    const uint64_t tile_bytes = tile_vecs << 4;
    // vectors between the last tile-size multiple and the first body vector of the destination
    auto lead_of = [&](const Seg &s) {
        return (uint64_t)((reinterpret_cast<uintptr_t>(s.dst + head_of(s.dst, s.bytes)) >> 4) % tile_vecs);
    };
    auto tiles_of = [&](const Seg &s) {
        const uint64_t nv = (s.bytes - head_of(s.dst, s.bytes)) >> 4;
        const uint64_t nt = (nv + lead_of(s) + tile_vecs - 1) / tile_vecs;
        return nt ? nt : (uint64_t)1;
    };
    uint64_t total = 0, longest = 0;
    plan.bytes = 0;
    for (const Seg &s : plan.segs) {
        const uint64_t nt = tiles_of(s);
        total += nt;
        if (nt > longest) longest = nt;
        plan.bytes += s.bytes;
    }
    // The launch is (tiles of the longest descriptor) x (descriptors); workgroups past
    // the end of a shorter descriptor leave at once.  If that would waste more than
    // 1/16 of the grid, or the grid would not fit, long segments are cut into pieces
    // of `limit` tiles (cuts fall on destination addresses that are multiples of the
    // tile size, so a later piece is itself a segment with an empty head and no lead).
    uint64_t limit = longest;
    const uint64_t nseg = plan.segs.size();
    if (nseg && (limit * nseg > total + total / 16 || limit > 0x7fffffffull)) {
        limit = 64;
        while (limit < 0x40000000ull && (total / limit + nseg) > 8192) limit <<= 1;
    }
    if (limit < longest) {
        std::vector<Seg> pieces;
        pieces.reserve((size_t)(total / limit + nseg));
        for (const Seg &s : plan.segs) {
            const uint32_t head = head_of(s.dst, s.bytes);
            const uint64_t first = head + limit * tile_bytes - (lead_of(s) << 4);   // bytes in the first piece
            if (s.bytes <= first) {
                pieces.push_back(s);
                continue;
            }
            pieces.push_back(Seg{s.src, s.dst, first, 0, 0});   // head and lead are filled in below
            for (uint64_t off = first; off < s.bytes; off += limit * tile_bytes) {
                const uint64_t n = s.bytes - off < limit * tile_bytes ? s.bytes - off : limit * tile_bytes;
                pieces.push_back(Seg{s.src + off, s.dst + off, n, 0, 0});
            }
        }
        plan.segs.swap(pieces);
    }
    uint64_t tiles = 0;
    longest = 0;
    for (Seg &s : plan.segs) {
        s.head = head_of(s.dst, s.bytes);
        s.lead = (uint32_t)lead_of(s);
        const uint64_t nt = tiles_of(s);
        tiles += nt;
        if (nt > longest) longest = nt;
    }
    plan.total_tiles = tiles;
    plan.max_tiles = (uint32_t)longest;
    return VCCL_OK;
}

template <int U, int POL, int T>
static void launch_threads(bool inl, bool fast, dim3 grid, hipStream_t stream, const CopyArgs &args) {
    const dim3 block(T);
    if (fast) {
        if (inl) copy_aligned_kernel<U, POL, true, T><<<grid, block, 0, stream>>>(args);
        else copy_aligned_kernel<U, POL, false, T><<<grid, block, 0, stream>>>(args);
    } else {
        if (inl) copy_segments_kernel<U, POL, true, T><<<grid, block, 0, stream>>>(args);
        else copy_segments_kernel<U, POL, false, T><<<grid, block, 0, stream>>>(args);
    }
}

template <int U, int POL>
static void launch_policy(bool inl, bool fast, int threads, dim3 grid, hipStream_t stream,
                          const CopyArgs &args) {
    if (threads == 64) launch_threads<U, POL, 64>(inl, fast, grid, stream, args);
    else if (threads == 128) launch_threads<U, POL, 128>(inl, fast, grid, stream, args);
    else launch_threads<U, POL, 256>(inl, fast, grid, stream, args);
}

template <int U>
static void launch_variant(int pol, bool inl, bool fast, int threads, dim3 grid, hipStream_t stream,
                           const CopyArgs &args) {
    if (pol == 2) launch_policy<U, 2>(inl, fast, threads, grid, stream, args);
    else if (pol == 1) launch_policy<U, 1>(inl, fast, threads, grid, stream, args);
    else launch_policy<U, 0>(inl, fast, threads, grid, stream, args);
}

int launch_copy(const CopyPlan &plan, const Options &opt, int cu_count, DescRing &ring,
                hipStream_t stream) {
    if (plan.segs.empty() || plan.total_tiles == 0) return VCCL_OK;
    CopyArgs args;
    args.table = nullptr;
    args.nseg = (uint32_t)plan.segs.size();
    args.pad = 0;
    DescSlot *slot = nullptr;
    struct SlotGuard {   // gives the staging slot back on every way out
        DescRing &ring;
        DescSlot *&slot;
        ~SlotGuard() {
            if (slot) ring.release(slot);
        }
    } guard{ring, slot};
    const bool inl = plan.segs.size() <= (size_t)kInlineSegs;
    if (inl) {
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
    // Full grid: one workgroup per tile.  Capped grid: cu_max_wg workgroups in all,
    // striding over descriptors and tiles.
    uint64_t gx = plan.max_tiles, gy = plan.segs.size();
    if (gy > 65535) gy = 65535;   // the kernel strides over descriptors beyond the grid
    const uint64_t cap = opt.cu_max_wg > 0 ? (uint64_t)opt.cu_max_wg
                                           : (opt.cu_wg_per_cu ? (uint64_t)cu_count * opt.cu_wg_per_cu : 0);
    if (cap && gx * gy > cap) {
        if (gy > cap) gy = cap;
        gx = cap / gy;
        if (gx < 1) gx = 1;
        if (gx > plan.max_tiles) gx = plan.max_tiles;
    }
    const dim3 grid((uint32_t)gx, (uint32_t)gy);
    const int nt = opt.cu_nontemporal;
    // A plan tiled for the all-aligned kernel must be run by it, on the full grid.
    const bool fast = plan.fast;
    if (fast && !(gx == plan.max_tiles && gy == plan.segs.size()))
        return fail(VCCL_ERR_UNSUPPORTED, "internal: a fast-path plan met a capped grid");
    switch (opt.cu_unroll) {
        case 1: launch_variant<1>(nt, inl, fast, plan.threads, grid, stream, args); break;
        case 2: launch_variant<2>(nt, inl, fast, plan.threads, grid, stream, args); break;
        case 4: launch_variant<4>(nt, inl, fast, plan.threads, grid, stream, args); break;
        case 8: launch_variant<8>(nt, inl, fast, plan.threads, grid, stream, args); break;
        case 16: launch_variant<16>(nt, inl, fast, plan.threads, grid, stream, args); break;
        default: return fail(VCCL_ERR_ARG, "cu_unroll %d is not one of 1,2,4,8,16", opt.cu_unroll);
    }
    VCCL_HIP(hipGetLastError());
    if (slot) VCCL_HIP(hipEventRecord(slot->done, stream));
    return VCCL_OK;
}

}  // namespace vccl
