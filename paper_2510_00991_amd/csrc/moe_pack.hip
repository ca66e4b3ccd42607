// MoE dispatch pack: make the rows bound for each destination rank contiguous
// before the AlltoAllv (token routing by AlltoAll, paper Section 2.1; dispatch
// phase, Section 6).  The (token, slot) pairs of a rank, in order p = t*K + k,
// are stably sorted by expert id; row j of the packed buffer is the row of the
// token of the j-th pair.  Stability makes the result unique, so it can be
// compared bit for bit.
//
// Four launches, all ranks at once (blockIdx.y = rank):
//   1 histogram   per-block expert counts (LDS atomics; counts do not depend on order)
//   2 scan        per expert: exclusive sum over blocks; across experts: exclusive
//                 sum with a wavefront shuffle scan  -> first row of (block, expert)
//   3 rank        wavefront ballot matching gives each pair its stable position
//   4 gather      a workgroup of 8 wavefronts per 2 KiB piece of a token's row: every
//                 wavefront loads the piece (the CU's vector cache serves the
//                 repeats, HBM is read once) and stores it to the destination of
//                 its own slot k (16 bytes per lane per access)
// The combine direction (vccl_moe_unpack) reuses launches 1-3 and replaces the
// gather by its inverse: row dest(t,k) of the packed buffer goes to row t*K+k.
// The per-rank form (vccl_moe_pack_per_rank: one row per token and destination
// rank) puts a key launch in front - rank of the expert for the first slot of a
// token that routes there, negative for repeats and bad ids - and a slot-to-row
// launch behind the same four.
#include "common.h"
#include "device_util.h"

namespace vccl {

constexpr int kPairsPerBlock = 2048;
constexpr int kMoeThreads = 256;
constexpr uint32_t kDropped = 0xffffffffu;
constexpr int kMaxExperts = 1024;

struct MoePtrs {       // device arrays of P pointers each, in one allocation
    const uint8_t *const *x;
    const int32_t *const *ids;      // sort keys: expert ids, or (per-rank form) rank keys in the scratch
    uint8_t *const *packed;
    const int32_t *const *ids_in;   // per-rank form: the caller's expert ids
    uint32_t *const *slot_row;      // per-rank form: the caller's slot-to-row maps (entries may be null)
    const uint64_t *capacity_rows;  // fused form: rows each destination rank's receive buffer holds
};
constexpr int kPtrArrays = 6;

// The two row buffers of every rank as a kernel argument (up to kInlineRanks ranks): a
// wavefront of the row-moving kernels then finds its buffers with one scalar load from
// the kernel-argument segment, instead of a load of the table's address followed by a
// load from the table - one memory round trip less in front of every row access, which
// measured 5 % of the gather's run time.  Must be the FIRST kernel argument: it is read
// in place through the kernel-argument pointer.
constexpr int kInlineRanks = 64;
struct RankPtrs {
    const uint8_t *x[kInlineRanks];
    uint8_t *packed[kInlineRanks];
};
template <bool INL>
__device__ __forceinline__ const u32x4 *rank_src(const MoePtrs &ptrs, uint32_t rank) {
    if (INL) {
        const RankPtrs *rp = reinterpret_cast<const RankPtrs *>((const void *)__builtin_amdgcn_kernarg_segment_ptr());
        return reinterpret_cast<const u32x4 *>(rp->x[rank]);
    }
    return reinterpret_cast<const u32x4 *>(ptrs.x[rank]);
}
template <bool INL>
__device__ __forceinline__ u32x4 *rank_dst(const MoePtrs &ptrs, uint32_t rank) {
    if (INL) {
        const RankPtrs *rp = reinterpret_cast<const RankPtrs *>((const void *)__builtin_amdgcn_kernarg_segment_ptr());
        return reinterpret_cast<u32x4 *>(rp->packed[rank]);
    }
    return reinterpret_cast<u32x4 *>(ptrs.packed[rank]);
}
constexpr int32_t kDuplicate = -1;   // rank key of a slot whose rank an earlier slot of the token already has
constexpr int32_t kBadId = -2;       // rank key of a slot whose expert id is out of range

__global__ __launch_bounds__(kMoeThreads) void moe_hist_kernel(MoePtrs ptrs, uint32_t npairs, int E,
                                                               uint32_t nblk, uint32_t *hist,
                                                               uint32_t *bad_ids) {
    __shared__ uint32_t h[kMaxExperts];
    const uint32_t rank = blockIdx.y, b = blockIdx.x;
    for (int e = threadIdx.x; e < E; e += kMoeThreads) h[e] = 0;
    __syncthreads();
    const int32_t *ids = ptrs.ids[rank];
    const uint32_t p0 = b * kPairsPerBlock;
    const uint32_t p1 = min(npairs, p0 + kPairsPerBlock);
    uint32_t bad = 0;
    for (uint32_t p = p0 + threadIdx.x; p < p1; p += kMoeThreads) {
        const int32_t e = ids[p];
        if (e >= 0 && e < E) atomicAdd(&h[e], 1u);
        else ++bad;
    }
    if (bad && bad_ids) atomicAdd(bad_ids, bad);
    __syncthreads();
    uint32_t *out = hist + ((size_t)rank * nblk + b) * (size_t)E;
    for (int e = threadIdx.x; e < E; e += kMoeThreads) out[e] = h[e];
}

// Per-rank form of the dispatch (one row per token and destination rank): the sort
// key of slot k is the destination rank of its expert if no earlier slot of the
// token routes to that rank, else kDuplicate; out-of-range ids give kBadId.  The
// index launches then see R "experts" and drop the negative keys.
__global__ __launch_bounds__(kMoeThreads) void moe_rank_keys_kernel(MoePtrs ptrs, uint32_t tokens, int K, int E,
                                                                    int experts_per_rank, int32_t *keys,
                                                                    uint32_t *bad_ids) {
    const uint32_t rank = blockIdx.y;
    const uint32_t t = blockIdx.x * kMoeThreads + threadIdx.x;
    if (t >= tokens) return;
    const int32_t *ids = ptrs.ids_in[rank] + (size_t)t * K;
    int32_t *out = keys + ((size_t)rank * tokens + t) * K;
    uint32_t bad = 0;
    for (int k = 0; k < K; ++k) {
        const int32_t e = ids[k];
        int32_t key;
        if (e < 0 || e >= E) {
            key = kBadId;
            ++bad;
        } else {
            key = e / experts_per_rank;
            for (int q = 0; q < k; ++q) {
                const int32_t eq = ids[q];
                if (eq >= 0 && eq < E && eq / experts_per_rank == key) {
                    key = kDuplicate;
                    break;
                }
            }
        }
        out[k] = key;
    }
    if (bad && bad_ids) atomicAdd(bad_ids, bad);
}

// slot_row[t*K + k] = packed row that serves slot k: its own if the slot carries the
// rank key, else the row of the earlier slot that carries the key of the same rank;
// kDropped for out-of-range ids.
__global__ __launch_bounds__(kMoeThreads) void moe_slot_row_kernel(MoePtrs ptrs, uint32_t tokens, int K,
                                                                   int experts_per_rank, const uint32_t *dest,
                                                                   uint32_t npairs) {
    const uint32_t rank = blockIdx.y;
    uint32_t *out = ptrs.slot_row[rank];
    const uint32_t t = blockIdx.x * kMoeThreads + threadIdx.x;
    if (!out || t >= tokens) return;
    const int32_t *keys = ptrs.ids[rank] + (size_t)t * K;
    const int32_t *ids = ptrs.ids_in[rank] + (size_t)t * K;
    const uint32_t *d = dest + (size_t)rank * npairs + (size_t)t * K;
    for (int k = 0; k < K; ++k) {
        uint32_t row = kDropped;
        if (keys[k] >= 0) {
            row = d[k];
        } else if (keys[k] == kDuplicate) {
            const int32_t r = ids[k] / experts_per_rank;
            for (int q = 0; q < k; ++q)
                if (keys[q] == r) row = d[q];
        }
        out[(size_t)t * K + k] = row;
    }
}

// Inclusive scan across the 64 lanes of a wavefront.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v, uint32_t lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(v, d, 64);
        if (lane >= (uint32_t)d) v += o;
    }
    return v;
}

__global__ __launch_bounds__(kMoeThreads) void moe_scan_kernel(int E, uint32_t nblk, uint32_t *hist,
                                                               uint64_t *counts) {
    __shared__ uint32_t wave_tot[kMoeThreads / 64];
    const uint32_t rank = blockIdx.x;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    uint32_t *hr = hist + (size_t)rank * nblk * (size_t)E;
    const int per = (E + kMoeThreads - 1) / kMoeThreads;   // consecutive experts per thread
    const int e0 = (int)tid * per;
    // pass 1, loads only (they do not depend on each other): pairs per expert
    uint32_t tot[kMaxExperts / kMoeThreads];
    uint32_t mine = 0;
    for (int j = 0; j < per; ++j) {
        const int e = e0 + j;
        uint32_t run = 0;
        if (e < E) {
#pragma unroll 8
            for (uint32_t b = 0; b < nblk; ++b) run += hr[(size_t)b * E + e];
            counts[(size_t)rank * E + e] = run;
        }
        tot[j] = run;
        mine += run;
    }
    // first row of each expert: exclusive sum across experts (lanes, then wavefronts)
    const uint32_t incl = wave_inclusive_scan(mine, lane);
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t base = incl - mine;
    for (uint32_t w = 0; w < wave; ++w) base += wave_tot[w];
    // pass 2: first row of each (block, expert) = the expert's first row + pairs in earlier blocks
    for (int j = 0; j < per; ++j) {
        const int e = e0 + j;
        if (e < E) {
            uint32_t run = base;
#pragma unroll 8
            for (uint32_t b = 0; b < nblk; ++b) {
                const uint32_t c = hr[(size_t)b * E + e];
                hr[(size_t)b * E + e] = run;
                run += c;
            }
        }
        base += tot[j];
    }
}

__global__ __launch_bounds__(kMoeThreads) void moe_rank_kernel(MoePtrs ptrs, uint32_t npairs, int E,
                                                               int ebits, uint32_t nblk,
                                                               const uint32_t *hist, uint32_t *dest) {
    __shared__ uint32_t next_row[kMaxExperts];
    const uint32_t rank = blockIdx.y, b = blockIdx.x;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t *off = hist + ((size_t)rank * nblk + b) * (size_t)E;
    for (int e = tid; e < E; e += kMoeThreads) next_row[e] = off[e];
    __syncthreads();
    const int32_t *ids = ptrs.ids[rank];
    uint32_t *drow = dest + (size_t)rank * npairs;
    const uint32_t p0 = b * kPairsPerBlock;
    const uint32_t p1 = min(npairs, p0 + kPairsPerBlock);
    const uint64_t lower_lanes = (1ull << lane) - 1ull;
    for (uint32_t base = p0; base < p1; base += kMoeThreads) {   // uniform trip count
        const uint32_t p = base + tid;
        const bool live = p < p1;
        const int32_t e = live ? ids[p] : -1;
        const bool ok = live && e >= 0 && e < E;
        // lanes of this wavefront that hold the same expert id
        uint64_t peers = __ballot(ok);
        for (int bit = 0; bit < ebits; ++bit) {
            const bool one = ((uint32_t)e >> bit) & 1u;
            const uint64_t m = __ballot(ok && one);
            peers &= one ? m : ~m;
        }
        const uint32_t before = (uint32_t)__popcll(peers & lower_lanes);
        const uint32_t group = (uint32_t)__popcll(peers);
        // the four wavefronts take their turn in pair order, which keeps the sort stable
        for (uint32_t w = 0; w < kMoeThreads / 64; ++w) {
            if (wave == w && ok) {
                const uint32_t start = next_row[e];
                drow[p] = start + before;
                if (before + 1 == group) next_row[e] = start + group;   // last peer advances
            }
            __syncthreads();
        }
        if (live && !ok) drow[p] = kDropped;
    }
}

// kRowVecs = 16-byte vectors a lane holds per pass over a row
template <int kRowVecs, bool NT>
__global__ __launch_bounds__(kMoeThreads) void moe_gather_kernel(MoePtrs ptrs, uint32_t tokens, int K,
                                                                 uint32_t row_vecs,
                                                                 const uint32_t *dest, uint32_t npairs) {
    const uint32_t rank = blockIdx.y;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t t = blockIdx.x * (kMoeThreads / 64) + (threadIdx.x >> 6);
    if (t >= tokens) return;
    const u32x4 *row = reinterpret_cast<const u32x4 *>(ptrs.x[rank]) + (size_t)t * row_vecs;
    u32x4 *out = reinterpret_cast<u32x4 *>(ptrs.packed[rank]);
    const uint32_t *d = dest + (size_t)rank * npairs + (size_t)t * K;
    for (uint32_t v0 = 0; v0 < row_vecs; v0 += 64u * kRowVecs) {
        u32x4 r[kRowVecs];
#pragma unroll
        for (int u = 0; u < kRowVecs; ++u) {
            const uint32_t v = v0 + u * 64u + lane;
            if (v < row_vecs) r[u] = __builtin_nontemporal_load(row + v);   // read once
        }
        for (int k = 0; k < K; ++k) {
            const uint32_t j = d[k];
            if (j == kDropped) continue;
            u32x4 *o = out + (size_t)j * row_vecs;
#pragma unroll
            for (int u = 0; u < kRowVecs; ++u) {
                const uint32_t v = v0 + u * 64u + lane;
                if (v < row_vecs) {
                    if (NT) __builtin_nontemporal_store(r[u], o + v);
                    else o[v] = r[u];
                }
            }
        }
    }
}

// Gather, shared-piece form.  Scattered 14 KiB-row writes cap HBM at about
// 5.5 TB/s whatever the workgroup shape; what this form removes is the long
// per-wavefront store sequence of the token-major kernel above (a wavefront there
// holds a row and issues K x 14 stores): here a wavefront loads at most two
// vectors per lane and stores them once.  Workgroup id = (token, piece, slot group);
// wavefront w of the workgroup serves slot k = 8*group + w.
constexpr int kPieceVecs = 128;   // 2 KiB
constexpr int kSlotWaves = 8;
// FULL: every piece is whole (row_vecs a multiple of kPieceVecs) and every slot group is
// full (K a multiple of kSlotWaves), so no wavefront has anything to test but "dropped".
// It is compiled for 7 wavefronts per SIMD instead of 8, which measured 1.43 against
// 1.46 ms on the 7.5 GB dispatch (6: 1.44 ms; 5 and fewer: 1.8 ms).
#define VCCL_GATHER_SHARED_BODY(FULL_)                                                                   \
    (void)by_value;                                                                                      \
    const uint32_t rank = blockIdx.y;                                                                    \
    const uint32_t t = per_token.div(blockIdx.x);                                                        \
    const uint32_t rem = blockIdx.x - t * per_token.d;                                                   \
    const uint32_t piece = kgroups.div(rem);                                                             \
    /* the wavefront index is the same in all lanes: say so, which makes the destination-row lookup a   \
       scalar load */                                                                                    \
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);                              \
    const uint32_t k = (rem - piece * kgroups.d) * kSlotWaves + wave;                                    \
    if (!(FULL_) && (t >= tokens || k >= (uint32_t)K)) return;                                           \
    const uint32_t v0 = piece * kPieceVecs + (threadIdx.x & 63u), v1 = v0 + 64u;                         \
    const u32x4 *row = rank_src<INL>(ptrs, rank) + (size_t)t * row_vecs;                                 \
    /* Row loads go out before the destination row is known (for a dropped pair they are wasted, which  \
       is rare).  Cached loads on purpose: the other 7 wavefronts read the same piece. */               \
    u32x4 r0 = {0, 0, 0, 0}, r1 = {0, 0, 0, 0};                                                          \
    if ((FULL_) || v0 < row_vecs) r0 = row[v0];                                                          \
    if ((FULL_) || v1 < row_vecs) r1 = row[v1];                                                          \
    const uint32_t j = dest[(size_t)rank * npairs + (size_t)t * K + k];                                  \
    /* (an empty statement that needs the loaded vectors: without it the compiler moves the row loads  \
       behind the test below, and every wavefront waits for its look-up before it asks for its row -   \
       1.74 instead of 1.43 ms on the 7.5 GB dispatch) */                                               \
    asm volatile("" ::"v"(r0), "v"(r1));                                                                 \
    if (j == kDropped) return;                                                                           \
    u32x4 *o = rank_dst<INL>(ptrs, rank) + (size_t)j * row_vecs;                                         \
    if ((FULL_) || v0 < row_vecs) {                                                                      \
        if (NT) __builtin_nontemporal_store(r0, o + v0);                                                 \
        else o[v0] = r0;                                                                                 \
    }                                                                                                    \
    if ((FULL_) || v1 < row_vecs) {                                                                      \
        if (NT) __builtin_nontemporal_store(r1, o + v1);                                                 \
        else o[v1] = r1;                                                                                 \
    }

template <bool NT, bool INL>
__global__ __launch_bounds__(kSlotWaves * 64) void moe_gather_shared_kernel(RankPtrs by_value, MoePtrs ptrs,
                                                                            uint32_t tokens, int K, uint32_t row_vecs,
                                                                            FastDiv per_token, FastDiv kgroups,
                                                                            const uint32_t *dest, uint32_t npairs) {
    VCCL_GATHER_SHARED_BODY(false)
}

template <bool NT, bool INL>
__global__ __launch_bounds__(kSlotWaves * 64) __attribute__((amdgpu_waves_per_eu(7, 7)))
void moe_gather_shared_full_kernel(RankPtrs by_value, MoePtrs ptrs, uint32_t tokens, int K, uint32_t row_vecs,
                                   FastDiv per_token, FastDiv kgroups, const uint32_t *dest, uint32_t npairs) {
    VCCL_GATHER_SHARED_BODY(true)
}
#undef VCCL_GATHER_SHARED_BODY

// Gather, piece-loop form: one single-wavefront workgroup per 2 KiB piece of a
// token's row loads the piece once and stores it for every slot that is not
// dropped.  This is the better shape when most slots are dropped, as in the
// per-rank form of the dispatch (a token reaches about 3 of 8 ranks on the
// measured routing): no wavefront is launched only to find its slot empty.
template <bool NT, bool INL>
__global__ __launch_bounds__(64) void moe_gather_piece_loop_kernel(RankPtrs by_value, MoePtrs ptrs, uint32_t tokens,
                                                                   int K, uint32_t row_vecs, FastDiv pieces,
                                                                   const uint32_t *dest, uint32_t npairs) {
    (void)by_value;
    const uint32_t rank = blockIdx.y;
    const uint32_t t = pieces.div(blockIdx.x);
    const uint32_t piece = blockIdx.x - t * pieces.d;
    if (t >= tokens) return;
    const uint32_t v0 = piece * kPieceVecs + threadIdx.x, v1 = v0 + 64u;
    const u32x4 *row = rank_src<INL>(ptrs, rank) + (size_t)t * row_vecs;
    u32x4 *out = rank_dst<INL>(ptrs, rank);
    u32x4 r0 = {0, 0, 0, 0}, r1 = {0, 0, 0, 0};
    if (v0 < row_vecs) r0 = __builtin_nontemporal_load(row + v0);   // read once
    if (v1 < row_vecs) r1 = __builtin_nontemporal_load(row + v1);
    const uint32_t *d = dest + (size_t)rank * npairs + (size_t)t * K;
    for (int k = 0; k < K; ++k) {
        const uint32_t j = d[k];
        if (j == kDropped) continue;
        u32x4 *o = out + (size_t)j * row_vecs;
        if (v0 < row_vecs) {
            if (NT) __builtin_nontemporal_store(r0, o + v0);
            else o[v0] = r0;
        }
        if (v1 < row_vecs) {
            if (NT) __builtin_nontemporal_store(r1, o + v1);
            else o[v1] = r1;
        }
    }
}

// Fused dispatch, layout step: from the per-expert counts of every source rank
// derive what the exchange after a pack would use - rows(s -> r), the four byte
// matrices - and, for the gather, delta[s][r] = first row of segment (s -> r) in
// recv[r] minus first row of rank r's block in s's packed order.  One workgroup;
// P*P is small.  status[1] is raised when a destination's rows exceed its capacity.
__global__ __launch_bounds__(kMoeThreads) void moe_fused_layout_kernel(const uint64_t *counts, int P, int E,
                                                                       int experts_per_rank, uint64_t row_bytes,
                                                                       const uint64_t *capacity_rows,
                                                                       uint64_t *layout, int64_t *delta,
                                                                       uint32_t *status) {
    uint64_t *sendcounts = layout, *sdispls = layout + (size_t)P * P;
    uint64_t *recvcounts = layout + 2 * (size_t)P * P, *rdispls = layout + 3 * (size_t)P * P;
    const int PP = P * P;
    for (int i = threadIdx.x; i < PP; i += kMoeThreads) {   // rows(s -> r), kept in sendcounts for now
        const int s = i / P, r = i - s * P;
        uint64_t rows = 0;
        for (int e = r * experts_per_rank; e < (r + 1) * experts_per_rank; ++e) rows += counts[(size_t)s * E + e];
        sendcounts[i] = rows;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < P; i += kMoeThreads) {    // prefix sums: over r for a sender, over s for a receiver
        uint64_t acc = 0;
        for (int r = 0; r < P; ++r) {
            sdispls[i * P + r] = acc;
            acc += sendcounts[i * P + r];
        }
        acc = 0;
        for (int s = 0; s < P; ++s) {
            rdispls[i * P + s] = acc;
            acc += sendcounts[s * P + i];
        }
        if (acc > capacity_rows[i] && status) atomicOr(status + 1, 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < PP; i += kMoeThreads) {
        const int s = i / P, r = i - s * P;
        delta[i] = (int64_t)rdispls[r * P + s] - (int64_t)sdispls[i];
        recvcounts[r * P + s] = sendcounts[i] * row_bytes;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < PP; i += kMoeThreads) {   // rows -> bytes
        sendcounts[i] *= row_bytes;
        sdispls[i] *= row_bytes;
        rdispls[i] *= row_bytes;
    }
}

// Fused dispatch, target step: where in which receive buffer the row of pair p goes
// (packed row -> expert's rank -> segment offset -> capacity), resolved once per pair
// into a pointer; null for a dropped pair or a row beyond the buffer's capacity.
// ptrs.packed holds the receive buffers here.
__global__ __launch_bounds__(kMoeThreads) void moe_pair_target_kernel(MoePtrs ptrs, uint32_t row_vecs,
                                                                      const uint32_t *dest, uint32_t npairs,
                                                                      int experts_per_rank, const int64_t *delta,
                                                                      int P, u32x4 **target) {
    const uint32_t rank = blockIdx.y;
    const uint32_t p = blockIdx.x * kMoeThreads + threadIdx.x;
    if (p >= npairs) return;
    u32x4 *row = nullptr;
    const uint32_t j = dest[(size_t)rank * npairs + p];
    if (j != kDropped) {
        const uint32_t to = (uint32_t)(ptrs.ids[rank][p] / experts_per_rank);
        const int64_t at = (int64_t)j + delta[(size_t)rank * P + to];
        if ((uint64_t)at < ptrs.capacity_rows[to])
            row = reinterpret_cast<u32x4 *>(ptrs.packed[to]) + (size_t)at * row_vecs;
    }
    target[(size_t)rank * npairs + p] = row;
}

// Fused dispatch, gather step: the shared-piece gather, except that the row of
// pair (t, k) goes straight into the receive buffer of the rank that hosts its
// expert, at the place the exchange would have put it.
#define VCCL_GATHER_FUSED_BODY(FULL_)                                                                    \
    (void)by_value;                                                                                      \
    const uint32_t rank = blockIdx.y;                                                                    \
    const uint32_t t = per_token.div(blockIdx.x);                                                        \
    const uint32_t rem = blockIdx.x - t * per_token.d;                                                   \
    const uint32_t piece = kgroups.div(rem);                                                             \
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);                              \
    const uint32_t k = (rem - piece * kgroups.d) * kSlotWaves + wave;                                    \
    if (!(FULL_) && (t >= tokens || k >= (uint32_t)K)) return;                                           \
    const uint32_t v0 = piece * kPieceVecs + (threadIdx.x & 63u), v1 = v0 + 64u;                         \
    const u32x4 *row = rank_src<INL>(ptrs, rank) + (size_t)t * row_vecs;                                 \
    u32x4 r0 = {0, 0, 0, 0}, r1 = {0, 0, 0, 0};                                                          \
    if ((FULL_) || v0 < row_vecs) r0 = row[v0];                                                          \
    if ((FULL_) || v1 < row_vecs) r1 = row[v1];                                                          \
    u32x4 *o = target[(size_t)rank * npairs + (size_t)t * K + k];                                        \
    asm volatile("" ::"v"(r0), "v"(r1));   /* keeps the row loads in front of the test, as above */      \
    if (!o) return;                                                                                      \
    if ((FULL_) || v0 < row_vecs) {                                                                      \
        if (NT) __builtin_nontemporal_store(r0, o + v0);                                                 \
        else o[v0] = r0;                                                                                 \
    }                                                                                                    \
    if ((FULL_) || v1 < row_vecs) {                                                                      \
        if (NT) __builtin_nontemporal_store(r1, o + v1);                                                 \
        else o[v1] = r1;                                                                                 \
    }

template <bool NT, bool INL>
__global__ __launch_bounds__(kSlotWaves * 64) void moe_gather_fused_kernel(RankPtrs by_value, MoePtrs ptrs,
                                                                           uint32_t tokens, int K, uint32_t row_vecs,
                                                                           FastDiv per_token, FastDiv kgroups,
                                                                           uint32_t npairs, u32x4 *const *target) {
    VCCL_GATHER_FUSED_BODY(false)
}

// whole pieces, whole slot groups, three workgroups per compute unit (see moe_gather_shared_full_kernel)
template <bool NT, bool INL>
__global__ __launch_bounds__(kSlotWaves * 64) __attribute__((amdgpu_waves_per_eu(7, 7)))
void moe_gather_fused_full_kernel(RankPtrs by_value, MoePtrs ptrs, uint32_t tokens, int K, uint32_t row_vecs,
                                  FastDiv per_token, FastDiv kgroups, uint32_t npairs, u32x4 *const *target) {
    VCCL_GATHER_FUSED_BODY(true)
}
#undef VCCL_GATHER_FUSED_BODY

// Inverse of the gather (combine direction): one workgroup per pair p = t*K + k
// copies the packed row that pair was sent to back to row p of `out`.  Writes sweep
// `out` front to back (the tight address window HBM likes), reads hop between
// expert regions in 14 KiB rows; every row is read once and written once.
__global__ __launch_bounds__(kMoeThreads) void moe_scatter_back_kernel(MoePtrs ptrs, uint32_t row_vecs,
                                                                       const uint32_t *dest,
                                                                       uint32_t npairs) {
    constexpr int kV = 4;
    const uint32_t rank = blockIdx.y;
    const uint32_t p = blockIdx.x;
    const uint32_t j = dest[(size_t)rank * npairs + p];
    if (j == kDropped) return;
    const u32x4 *row = reinterpret_cast<const u32x4 *>(ptrs.x[rank]) + (size_t)j * row_vecs;   // packed side
    u32x4 *o = reinterpret_cast<u32x4 *>(ptrs.packed[rank]) + (size_t)p * row_vecs;          // token order
    for (uint32_t v0 = 0; v0 < row_vecs; v0 += (uint32_t)kMoeThreads * kV) {
        u32x4 r[kV];
#pragma unroll
        for (int u = 0; u < kV; ++u) {
            const uint32_t v = v0 + u * kMoeThreads + threadIdx.x;
            if (v < row_vecs) r[u] = __builtin_nontemporal_load(row + v);
        }
#pragma unroll
        for (int u = 0; u < kV; ++u) {
            const uint32_t v = v0 + u * kMoeThreads + threadIdx.x;
            if (v < row_vecs) __builtin_nontemporal_store(r[u], o + v);
        }
    }
}

// Combine direction, tile form: one single-wavefront workgroup per 1 KiB tile of
// `out`, in address order - the launch shape of the exchange copy kernel, which
// HBM serves best; the reads hop between expert regions row by row.
template <int POL, int TILES, bool INL>
__global__ __launch_bounds__(64) void moe_scatter_back_tiles_kernel(RankPtrs by_value, MoePtrs ptrs, uint32_t row_vecs,
                                                                    FastDiv groups_per_row, const uint32_t *dest,
                                                                    uint32_t npairs) {
    (void)by_value;
    const uint32_t rank = blockIdx.y;
    const uint32_t p = groups_per_row.div(blockIdx.x);
    const uint32_t v0 = (blockIdx.x - p * groups_per_row.d) * (64u * TILES);
    if (p >= npairs) return;
    const uint32_t j = dest[(size_t)rank * npairs + p];
    if (j == kDropped) return;
    const u32x4 *row = rank_src<INL>(ptrs, rank) + (size_t)j * row_vecs + v0;   // packed side
    const TileDst<POL> o(rank_dst<INL>(ptrs, rank) + (size_t)p * row_vecs + v0);
    u32x4 r[TILES];
#pragma unroll
    for (int u = 0; u < TILES; ++u)
        if (v0 + u * 64u + threadIdx.x < row_vecs) r[u] = ld16<POL>(row + u * 64u + threadIdx.x);
#pragma unroll
    for (int u = 0; u < TILES; ++u)
        if (v0 + u * 64u + threadIdx.x < row_vecs) o.store(u * 64u + threadIdx.x, r[u]);
}

// Fused combine: the inverse exchange and the un-permute in one pass.  Row p = t*K + k
// of out[s] comes straight from the place in back[r] (r = rank of the pair's expert)
// where the fused dispatch - or pack + exchange - had put the pair's row.  A first
// launch resolves, per pair, where that row is (destination row -> expert's rank ->
// segment offset -> capacity: four dependent look-ups) into one pointer, null for a
// pair that is dropped or beyond the buffer's capacity; the tile kernel then has
// the same short chain as the un-permute kernel above: one look-up, load, store.
__global__ __launch_bounds__(kMoeThreads) void moe_pair_source_kernel(MoePtrs ptrs, uint32_t row_vecs,
                                                                      const uint32_t *dest, uint32_t npairs,
                                                                      int experts_per_rank, const int64_t *delta,
                                                                      int P, const u32x4 **source) {
    const uint32_t rank = blockIdx.y;
    const uint32_t p = blockIdx.x * kMoeThreads + threadIdx.x;
    if (p >= npairs) return;
    const u32x4 *row = nullptr;
    const uint32_t j = dest[(size_t)rank * npairs + p];
    if (j != kDropped) {
        const uint32_t from = (uint32_t)(ptrs.ids[rank][p] / experts_per_rank);
        const int64_t at = (int64_t)j + delta[(size_t)rank * P + from];
        if ((uint64_t)at < ptrs.capacity_rows[from])
            row = reinterpret_cast<const u32x4 *>(ptrs.x[from]) + (size_t)at * row_vecs;
    }
    source[(size_t)rank * npairs + p] = row;
}

// ptrs.packed holds the P outputs; 1 KiB single-wavefront tiles in output order.
template <int POL, bool INL>
__global__ __launch_bounds__(64) void moe_combine_fused_kernel(RankPtrs by_value, MoePtrs ptrs, uint32_t row_vecs,
                                                               FastDiv tiles_per_row, uint32_t npairs,
                                                               const u32x4 *const *source) {
    (void)by_value;
    const uint32_t rank = blockIdx.y;
    const uint32_t p = tiles_per_row.div(blockIdx.x);
    const uint32_t v0 = (blockIdx.x - p * tiles_per_row.d) * 64u;
    if (p >= npairs) return;
    const u32x4 *row = source[(size_t)rank * npairs + p];
    if (!row) return;
    const TileDst<POL> o(rank_dst<INL>(ptrs, rank) + (size_t)p * row_vecs + v0);
    if (v0 + threadIdx.x < row_vecs) o.store(threadIdx.x, ld16<POL>(row + v0 + threadIdx.x));
}

void MoeScratch::destroy() {
    if (done) {
        (void)hipEventSynchronize(done);
        (void)hipEventDestroy(done);
        done = nullptr;
    }
    if (hist) (void)hipFree(hist);
    if (ptrs) (void)hipFree(ptrs);
    if (ptrs_host) (void)hipHostFree(ptrs_host);
    hist = nullptr;
    ptrs = nullptr;
    ptrs_host = nullptr;
    hist_n = ptrs_n = 0;
}

// ---- scratch of the entry point that allocates nothing ------------------------
// vccl_moe_pack_noalloc keeps its index data (histograms, destination rows, counts,
// the table of rank pointers) in this file-scope array instead of allocated memory.
// Host code never uses the array's name as an address: its device address is asked
// for once per device (moe_static_scratch_init) and kept in g_static_scratch.
constexpr size_t kStaticScratchBytes = 8u << 20;
constexpr int kStaticMaxRanks = 16;
constexpr int kStaticMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static void *g_static_scratch[kStaticMaxDevices] = {};
static std::mutex g_static_mu;

int moe_static_scratch_init(int device) {
    if (device < 0 || device >= kStaticMaxDevices)
        return fail(VCCL_ERR_UNSUPPORTED, "device %d is beyond the %d devices the static scratch is kept for", device,
                    kStaticMaxDevices);
    std::lock_guard<std::mutex> lk(g_static_mu);
    if (g_static_scratch[device]) return VCCL_OK;
    void *ptr = nullptr;
    VCCL_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));   // the current device's copy of the array
    if (!ptr) return fail(VCCL_ERR_HIP, "hipGetSymbolAddress gave a null address for the static scratch");
    g_static_scratch[device] = ptr;
    return VCCL_OK;
}

constexpr int kTableRanks = 64;   // ranks whose pointer table fits a kernel argument
struct PtrBlock {   // the rank-pointer table as a kernel argument
    void *p[kPtrArrays * kTableRanks];
};
static_assert(sizeof(PtrBlock) <= 3072 && kStaticMaxRanks <= kTableRanks, "kernel-argument budget");
__global__ __launch_bounds__(kMoeThreads) void moe_store_ptrs_kernel(PtrBlock blk, void **table, int n) {
    const int i = blockIdx.x * kMoeThreads + threadIdx.x;
    if (i < n) table[i] = blk.p[i];
}

// Where the index data of one call lives: `words` holds histograms, destination rows,
// rank keys, counts and the caller's extra room, `ptrs` the device table of
// kPtrArrays x P rank pointers.
struct MoeWork {
    uint32_t *words;
    void **ptrs;
};

// 32-bit words one call needs (see moe_index_phase for the layout).
static size_t moe_words_needed(int P, int tokens, int topk, int num_experts, int experts_per_rank,
                               size_t extra_words) {
    const bool per_rank = experts_per_rank > 0;
    const int nkeys = per_rank ? num_experts / experts_per_rank : num_experts;
    const uint32_t npairs = (uint32_t)tokens * (uint32_t)topk;
    const uint32_t nblk = npairs ? (npairs + kPairsPerBlock - 1) / kPairsPerBlock : 1;
    const size_t hist_n = (size_t)P * nblk * (size_t)nkeys;
    const size_t counts_words = 2 * (size_t)P * nkeys;
    const size_t keys_words = per_rank ? (size_t)P * npairs : 0;
    // histograms, destination rows, rank keys, counts (8-byte aligned), caller's extra (8-byte aligned)
    return hist_n + (size_t)P * npairs + keys_words + counts_words + 2 + extra_words + 2;
}

// Row of the rank-pointer table: what every kernel of the MoE path reads its buffers from.
static void moe_fill_ptr_table(void **tbl, uint32_t *words, const void *const *a, const int32_t *const *ids,
                               int P, int tokens, int topk, int num_experts, int experts_per_rank,
                               uint32_t *const *slot_row, void *const *b, const uint64_t *capacity_rows) {
    const bool per_rank = experts_per_rank > 0;
    const int nkeys = per_rank ? num_experts / experts_per_rank : num_experts;
    const uint32_t npairs = (uint32_t)tokens * (uint32_t)topk;
    const uint32_t nblk = npairs ? (npairs + kPairsPerBlock - 1) / kPairsPerBlock : 1;
    const size_t hist_n = (size_t)P * nblk * (size_t)nkeys;
    int32_t *keys = reinterpret_cast<int32_t *>(words + hist_n + (size_t)P * npairs);
    for (int s = 0; s < P; ++s) {
        tbl[s] = const_cast<void *>(a[s]);
        tbl[P + s] = per_rank ? static_cast<void *>(keys + (size_t)s * npairs)
                              : static_cast<void *>(const_cast<int32_t *>(ids[s]));
        tbl[2 * P + s] = b[s];
        tbl[3 * P + s] = const_cast<int32_t *>(ids[s]);
        tbl[4 * P + s] = slot_row ? slot_row[s] : nullptr;
        tbl[5 * P + s] = reinterpret_cast<void *>((uintptr_t)(capacity_rows ? capacity_rows[s] : 0));
    }
}

// Launches 1-3: per-pair destination rows in `w.words`; the pointer table `w.ptrs` is
// already on its way on `stream`.  experts_per_rank > 0 selects the per-rank form: the
// sort keys are computed into the scratch from the caller's ids and `num_experts`
// counts ranks from there on.
static int moe_index_launches(const MoeWork &w, int P, int tokens, int topk, int num_experts,
                              int experts_per_rank, uint64_t *counts_dev, uint32_t *bad_ids_dev,
                              hipStream_t stream, MoePtrs *ptrs_out, uint32_t **dest_out,
                              uint64_t **counts_out, uint64_t **extra_out) {
    const bool per_rank = experts_per_rank > 0;
    const int nkeys = per_rank ? num_experts / experts_per_rank : num_experts;   // sort-key range
    const uint32_t npairs = (uint32_t)tokens * (uint32_t)topk;
    const uint32_t nblk = npairs ? (npairs + kPairsPerBlock - 1) / kPairsPerBlock : 1;
    const size_t hist_n = (size_t)P * nblk * (size_t)nkeys;
    const size_t keys_words = per_rank ? (size_t)P * npairs : 0;
    uint32_t *hist = w.words;
    uint32_t *dest = w.words + hist_n;
    int32_t *keys = reinterpret_cast<int32_t *>(dest + (size_t)P * npairs);
    MoePtrs ptrs;
    ptrs.x = reinterpret_cast<const uint8_t *const *>(w.ptrs);
    ptrs.ids = reinterpret_cast<const int32_t *const *>(w.ptrs + P);
    ptrs.packed = reinterpret_cast<uint8_t *const *>(w.ptrs + 2 * P);
    ptrs.ids_in = reinterpret_cast<const int32_t *const *>(w.ptrs + 3 * P);
    ptrs.slot_row = reinterpret_cast<uint32_t *const *>(w.ptrs + 4 * P);
    ptrs.capacity_rows = reinterpret_cast<const uint64_t *>(w.ptrs + 5 * P);
    static_assert(sizeof(void *) == sizeof(uint64_t), "capacities travel in pointer-sized slots");
    uint64_t *counts_scratch =
        reinterpret_cast<uint64_t *>((reinterpret_cast<uintptr_t>(keys + keys_words) + 7u) & ~(uintptr_t)7u);
    if (!counts_dev) counts_dev = counts_scratch;   // the caller does not want the counts
    if (counts_out) *counts_out = counts_dev;
    if (extra_out) *extra_out = counts_scratch + (size_t)P * nkeys;
    int ebits = 0;
    while ((1 << ebits) < nkeys) ++ebits;
    if (per_rank && tokens) {
        // out-of-range ids are counted here; the histogram then sees them as negative keys
        moe_rank_keys_kernel<<<dim3(((uint32_t)tokens + kMoeThreads - 1) / kMoeThreads, P), dim3(kMoeThreads), 0,
                               stream>>>(ptrs, (uint32_t)tokens, topk, num_experts, experts_per_rank, keys,
                                         bad_ids_dev);
        VCCL_HIP(hipGetLastError());
        bad_ids_dev = nullptr;
    }
    moe_hist_kernel<<<dim3(nblk, P), dim3(kMoeThreads), 0, stream>>>(ptrs, npairs, nkeys, nblk, hist,
                                                                    bad_ids_dev);
    VCCL_HIP(hipGetLastError());
    moe_scan_kernel<<<dim3(P), dim3(kMoeThreads), 0, stream>>>(nkeys, nblk, hist, counts_dev);
    VCCL_HIP(hipGetLastError());
    if (npairs) {
        moe_rank_kernel<<<dim3(nblk, P), dim3(kMoeThreads), 0, stream>>>(ptrs, npairs, nkeys, ebits, nblk,
                                                                        hist, dest);
        VCCL_HIP(hipGetLastError());
    }
    *ptrs_out = ptrs;
    *dest_out = dest;
    return VCCL_OK;
}

// The allocating entry points: grow the library-owned scratch as needed, put the
// pointer table on the device, then launches 1-3.  `a` / `b` are the two
// row buffers of every rank in the roles (read side, written side) of launch 4.
static int moe_index_phase(MoeScratch &sc, const void *const *a, const int32_t *const *ids, int P,
                           int tokens, int topk, int num_experts, int experts_per_rank,
                           uint32_t *const *slot_row, void *const *b, const uint64_t *capacity_rows,
                           size_t extra_words, uint64_t *counts_dev, uint32_t *bad_ids_dev,
                           hipStream_t stream, MoePtrs *ptrs_out, uint32_t **dest_out,
                           uint64_t **counts_out = nullptr, uint64_t **extra_out = nullptr) {
    const size_t need = moe_words_needed(P, tokens, topk, num_experts, experts_per_rank, extra_words);
    if (!sc.done) VCCL_HIP(hipEventCreateWithFlags(&sc.done, hipEventDisableTiming));
    // The scratch is shared between calls.  Up to kTableRanks ranks the pointer table
    // reaches the device as a kernel argument, so the only thing a new call has to wait
    // for is the previous call's kernels, and the stream can do that waiting: calls
    // follow each other without the host in between.  The host waits only when memory
    // is about to be reallocated, or (more ranks) when the pinned staging is reused.
    const bool grow = need > sc.hist_n || (size_t)kPtrArrays * P > sc.ptrs_n;
    const bool by_kernel = P <= kTableRanks;
    if (grow || !by_kernel) VCCL_HIP(hipEventSynchronize(sc.done));
    else VCCL_HIP(hipStreamWaitEvent(stream, sc.done, 0));
    if (need > sc.hist_n) {
        if (sc.hist) VCCL_HIP(hipFree(sc.hist));
        sc.hist = nullptr;
        sc.hist_n = 0;
        VCCL_HIP(hipMalloc((void **)&sc.hist, need * sizeof(uint32_t)));
        sc.hist_n = need;
    }
    if ((size_t)kPtrArrays * P > sc.ptrs_n) {
        if (sc.ptrs) VCCL_HIP(hipFree(sc.ptrs));
        if (sc.ptrs_host) VCCL_HIP(hipHostFree(sc.ptrs_host));
        sc.ptrs = nullptr;
        sc.ptrs_host = nullptr;
        sc.ptrs_n = 0;
        VCCL_HIP(hipMalloc((void **)&sc.ptrs, (size_t)kPtrArrays * P * sizeof(void *)));
        VCCL_HIP(hipHostMalloc((void **)&sc.ptrs_host, (size_t)kPtrArrays * P * sizeof(void *), hipHostMallocDefault));
        sc.ptrs_n = (size_t)kPtrArrays * P;
    }
    if (by_kernel) {
        PtrBlock blk;
        moe_fill_ptr_table(blk.p, sc.hist, a, ids, P, tokens, topk, num_experts, experts_per_rank, slot_row, b,
                           capacity_rows);
        const int n = kPtrArrays * P;
        for (int i = n; i < kPtrArrays * kTableRanks; ++i) blk.p[i] = nullptr;
        moe_store_ptrs_kernel<<<dim3((n + kMoeThreads - 1) / kMoeThreads), dim3(kMoeThreads), 0, stream>>>(blk, sc.ptrs, n);
        VCCL_HIP(hipGetLastError());
    } else {
        moe_fill_ptr_table(sc.ptrs_host, sc.hist, a, ids, P, tokens, topk, num_experts, experts_per_rank, slot_row,
                           b, capacity_rows);
        VCCL_HIP(hipMemcpyAsync(sc.ptrs, sc.ptrs_host, (size_t)kPtrArrays * P * sizeof(void *),
                                hipMemcpyHostToDevice, stream));
    }
    const MoeWork w{sc.hist, sc.ptrs};
    return moe_index_launches(w, P, tokens, topk, num_experts, experts_per_rank, counts_dev, bad_ids_dev, stream,
                              ptrs_out, dest_out, counts_out, extra_out);
}

// The rank buffers as a kernel argument (read side `a`, written side `b`; either may be
// null when a kernel does not use that side); false when there are too many ranks.
static bool rank_ptrs_inline(RankPtrs &rp, const void *const *a, void *const *b, int P) {
    if (P > kInlineRanks) return false;
    for (int s = 0; s < kInlineRanks; ++s) {
        rp.x[s] = (s < P && a) ? static_cast<const uint8_t *>(a[s]) : nullptr;
        rp.packed[s] = (s < P && b) ? static_cast<uint8_t *>(b[s]) : nullptr;
    }
    return true;
}

// Launch 4 of the pack: the row gather in the selected form.
static int moe_launch_gather(const MoePtrs &ptrs, const void *const *x, void *const *packed, const uint32_t *dest,
                             int P, int tokens, int topk, uint64_t row_bytes, int experts_per_rank,
                             int gather_variant, int gather_full, hipStream_t stream) {
    RankPtrs rp;
    const bool inl = rank_ptrs_inline(rp, x, packed, P);
    const uint32_t npairs = (uint32_t)tokens * (uint32_t)topk;
    const uint32_t tok_blocks = ((uint32_t)tokens + kMoeThreads / 64 - 1) / (kMoeThreads / 64);
    const dim3 g(tok_blocks, P), b(kMoeThreads);
    const uint32_t rv = (uint32_t)(row_bytes >> 4);
    const uint32_t pieces = (rv + kPieceVecs - 1) / kPieceVecs;
    const uint32_t kgroups = ((uint32_t)topk + kSlotWaves - 1) / kSlotWaves;
    const uint64_t shared_grid = (uint64_t)tokens * pieces * kgroups;
    if ((gather_variant == 208 || gather_variant == 308) && shared_grid > 0x7fffffffull) gather_variant = 116;
    // per-rank form: most slots are dropped, the piece-loop kernel wastes no wavefront on them
    if (experts_per_rank > 0 && (gather_variant == 208 || gather_variant == 308)) gather_variant += 200;
    const uint64_t loop_grid = (uint64_t)tokens * pieces;
    if ((gather_variant == 408 || gather_variant == 508) && loop_grid > 0x7fffffffull) gather_variant = 116;
    const dim3 gl((uint32_t)loop_grid, P), bl(64);
    const dim3 gs((uint32_t)shared_grid, P), bs(kSlotWaves * 64);
    const FastDiv dpieces(pieces), dkgroups(kgroups), dper_token(pieces * kgroups);
    const uint32_t ut = (uint32_t)tokens;
    // whole pieces and whole slot groups only (gather_full = 0 keeps the checked kernel, for tests)
    const bool full = gather_full && rv % kPieceVecs == 0 && topk % kSlotWaves == 0;
#define VCCL_GATHER(KERNEL, NT, GRID, BLOCK, LDS, ...)                                            \
    do {                                                                                          \
        if (inl) KERNEL<NT, true><<<GRID, BLOCK, LDS, stream>>>(rp, ptrs, __VA_ARGS__);            \
        else KERNEL<NT, false><<<GRID, BLOCK, LDS, stream>>>(rp, ptrs, __VA_ARGS__);               \
    } while (0)
    switch (gather_variant) {
        case 408: VCCL_GATHER(moe_gather_piece_loop_kernel, true, gl, bl, 0, ut, topk, rv, dpieces, dest, npairs); break;
        case 508: VCCL_GATHER(moe_gather_piece_loop_kernel, false, gl, bl, 0, ut, topk, rv, dpieces, dest, npairs); break;
        case 208:
            if (full) VCCL_GATHER(moe_gather_shared_full_kernel, true, gs, bs, 0, ut, topk, rv, dper_token, dkgroups, dest, npairs);
            else VCCL_GATHER(moe_gather_shared_kernel, true, gs, bs, 0, ut, topk, rv, dper_token, dkgroups, dest, npairs);
            break;
        case 308:
            if (full) VCCL_GATHER(moe_gather_shared_full_kernel, false, gs, bs, 0, ut, topk, rv, dper_token, dkgroups, dest, npairs);
            else VCCL_GATHER(moe_gather_shared_kernel, false, gs, bs, 0, ut, topk, rv, dper_token, dkgroups, dest, npairs);
            break;
        case 4: moe_gather_kernel<4, true><<<g, b, 0, stream>>>(ptrs, (uint32_t)tokens, topk, rv, dest, npairs); break;
        case 16: moe_gather_kernel<16, true><<<g, b, 0, stream>>>(ptrs, (uint32_t)tokens, topk, rv, dest, npairs); break;
        case 108: moe_gather_kernel<8, false><<<g, b, 0, stream>>>(ptrs, (uint32_t)tokens, topk, rv, dest, npairs); break;
        case 116: moe_gather_kernel<16, false><<<g, b, 0, stream>>>(ptrs, (uint32_t)tokens, topk, rv, dest, npairs); break;
        default: moe_gather_kernel<8, true><<<g, b, 0, stream>>>(ptrs, (uint32_t)tokens, topk, rv, dest, npairs); break;
    }
#undef VCCL_GATHER
    VCCL_HIP(hipGetLastError());
    return VCCL_OK;
}

// The pack without any allocation: index data and pointer table in the static scratch.
// No event guards the scratch: calls that overlap on one device race (documented).
int launch_moe_pack_noalloc(int device, const void *const *x, const int32_t *const *ids, int P, int tokens,
                            int topk, uint64_t row_bytes, int num_experts, void *const *packed,
                            uint64_t *counts_dev, uint32_t *bad_ids_dev, int gather_variant, int gather_full,
                            hipStream_t stream) {
    if (device < 0 || device >= kStaticMaxDevices || !g_static_scratch[device])
        return fail(VCCL_ERR_NOT_INIT, "the static scratch of device %d has not been set up (vccl_init does it)", device);
    if (P > kStaticMaxRanks)
        return fail(VCCL_ERR_UNSUPPORTED, "vccl_moe_pack_noalloc takes at most %d ranks, got %d", kStaticMaxRanks, P);
    constexpr size_t kTableBytes = ((sizeof(PtrBlock) + 255u) / 256u) * 256u;
    const size_t need = moe_words_needed(P, tokens, topk, num_experts, 0, 0);
    if (kTableBytes + need * sizeof(uint32_t) > kStaticScratchBytes)
        return fail(VCCL_ERR_UNSUPPORTED,
                    "vccl_moe_pack_noalloc: P = %d, tokens = %d, topk = %d, num_experts = %d need %zu bytes of index "
                    "data, the static scratch holds %zu (use vccl_moe_pack)", P, tokens, topk, num_experts,
                    kTableBytes + need * sizeof(uint32_t), kStaticScratchBytes);
    unsigned char *base = static_cast<unsigned char *>(g_static_scratch[device]);
    const MoeWork w{reinterpret_cast<uint32_t *>(base + kTableBytes), reinterpret_cast<void **>(base)};
    PtrBlock blk;
    moe_fill_ptr_table(blk.p, w.words, x, ids, P, tokens, topk, num_experts, 0, nullptr, packed, nullptr);
    const int n = kPtrArrays * P;
    for (int i = n; i < kPtrArrays * kTableRanks; ++i) blk.p[i] = nullptr;
    moe_store_ptrs_kernel<<<dim3((n + kMoeThreads - 1) / kMoeThreads), dim3(kMoeThreads), 0, stream>>>(blk, w.ptrs, n);
    VCCL_HIP(hipGetLastError());
    // Nothing in the scratch has to start at zero: every histogram word, destination row
    // and count this call reads is written by this call first.
    MoePtrs ptrs;
    uint32_t *dest = nullptr;
    int rc = moe_index_launches(w, P, tokens, topk, num_experts, 0, counts_dev, bad_ids_dev, stream, &ptrs, &dest,
                                nullptr, nullptr);
    if (rc) return rc;
    if ((uint32_t)tokens * (uint32_t)topk)
        return moe_launch_gather(ptrs, x, packed, dest, P, tokens, topk, row_bytes, 0, gather_variant, gather_full, stream);
    return VCCL_OK;
}

int launch_moe_pack(MoeScratch &sc, const void *const *x, const int32_t *const *ids, int P, int tokens,
                    int topk, uint64_t row_bytes, int num_experts, int experts_per_rank,
                    void *const *packed, uint64_t *counts_dev, uint64_t *counts_host,
                    uint32_t *const *slot_row, uint32_t *bad_ids_dev, int gather_variant, int gather_full,
                    hipStream_t stream) {
    const uint32_t npairs = (uint32_t)tokens * (uint32_t)topk;
    std::lock_guard<std::mutex> lk(sc.mu);
    MoePtrs ptrs;
    uint32_t *dest = nullptr;
    int rc = moe_index_phase(sc, x, ids, P, tokens, topk, num_experts, experts_per_rank, slot_row, packed,
                             nullptr, 0, counts_dev, bad_ids_dev, stream, &ptrs, &dest);
    if (rc) return rc;
    if (npairs) {
        rc = moe_launch_gather(ptrs, x, packed, dest, P, tokens, topk, row_bytes, experts_per_rank, gather_variant,
                               gather_full, stream);
        if (rc) return rc;
        if (experts_per_rank > 0 && slot_row) {
            moe_slot_row_kernel<<<dim3(((uint32_t)tokens + kMoeThreads - 1) / kMoeThreads, P), dim3(kMoeThreads),
                                  0, stream>>>(ptrs, (uint32_t)tokens, topk, experts_per_rank, dest, npairs);
            VCCL_HIP(hipGetLastError());
        }
    }
    const int ncounts = experts_per_rank > 0 ? num_experts / experts_per_rank : num_experts;
    if (counts_host)
        VCCL_HIP(hipMemcpyAsync(counts_host, counts_dev, (size_t)P * ncounts * sizeof(uint64_t),
                                hipMemcpyDeviceToHost, stream));
    VCCL_HIP(hipEventRecord(sc.done, stream));
    return VCCL_OK;
}

int launch_moe_dispatch_fused(MoeScratch &sc, const void *const *x, const int32_t *const *ids, int P, int tokens,
                              int topk, uint64_t row_bytes, int num_experts, int experts_per_rank,
                              void *const *recv, const uint64_t *capacity_rows, uint64_t *counts_dev,
                              uint64_t *layout_dev, uint64_t *layout_host, uint32_t *status_dev,
                              int gather_full, hipStream_t stream) {
    const uint32_t npairs = (uint32_t)tokens * (uint32_t)topk;
    const uint32_t rv = (uint32_t)(row_bytes >> 4);
    const uint32_t pieces = (rv + kPieceVecs - 1) / kPieceVecs;
    const uint32_t kgroups = ((uint32_t)topk + kSlotWaves - 1) / kSlotWaves;
    const uint64_t grid = (uint64_t)tokens * pieces * kgroups;
    if (grid > 0x7fffffffull)
        return fail(VCCL_ERR_UNSUPPORTED, "tokens x row pieces x slot groups = %llu exceeds the launch grid",
                    (unsigned long long)grid);
    std::lock_guard<std::mutex> lk(sc.mu);
    MoePtrs ptrs;
    uint32_t *dest = nullptr;
    uint64_t *counts = nullptr, *extra = nullptr;
    // room after the counts: delta [P][P] (int64), one target pointer per pair
    int rc = moe_index_phase(sc, x, ids, P, tokens, topk, num_experts, 0, nullptr, recv, capacity_rows,
                             2 * ((size_t)P * P + (size_t)P * npairs), counts_dev, status_dev, stream, &ptrs, &dest,
                             &counts, &extra);
    if (rc) return rc;
    int64_t *delta = reinterpret_cast<int64_t *>(extra);
    u32x4 **target = reinterpret_cast<u32x4 **>(extra + (size_t)P * P);
    moe_fused_layout_kernel<<<dim3(1), dim3(kMoeThreads), 0, stream>>>(counts, P, num_experts, experts_per_rank,
                                                                      row_bytes, ptrs.capacity_rows, layout_dev,
                                                                      delta, status_dev);
    VCCL_HIP(hipGetLastError());
    if (npairs) {
        moe_pair_target_kernel<<<dim3((npairs + kMoeThreads - 1) / kMoeThreads, P), dim3(kMoeThreads), 0, stream>>>(
            ptrs, rv, dest, npairs, experts_per_rank, delta, P, target);
        VCCL_HIP(hipGetLastError());
        RankPtrs rp;
        const FastDiv dkgroups(kgroups), dper_token(pieces * kgroups);
        const dim3 gg((uint32_t)grid, P), gb(kSlotWaves * 64);
        const bool inl = rank_ptrs_inline(rp, x, nullptr, P);
        const bool full = gather_full && rv % kPieceVecs == 0 && topk % kSlotWaves == 0;
        const uint32_t ut = (uint32_t)tokens;
        if (full && inl) moe_gather_fused_full_kernel<true, true><<<gg, gb, 0, stream>>>(rp, ptrs, ut, topk, rv, dper_token, dkgroups, npairs, target);
        else if (full) moe_gather_fused_full_kernel<true, false><<<gg, gb, 0, stream>>>(rp, ptrs, ut, topk, rv, dper_token, dkgroups, npairs, target);
        else if (inl) moe_gather_fused_kernel<true, true><<<gg, gb, 0, stream>>>(rp, ptrs, ut, topk, rv, dper_token, dkgroups, npairs, target);
        else moe_gather_fused_kernel<true, false><<<gg, gb, 0, stream>>>(rp, ptrs, ut, topk, rv, dper_token, dkgroups, npairs, target);
        VCCL_HIP(hipGetLastError());
    }
    if (layout_host)
        VCCL_HIP(hipMemcpyAsync(layout_host, layout_dev, 4 * (size_t)P * P * sizeof(uint64_t),
                                hipMemcpyDeviceToHost, stream));
    VCCL_HIP(hipEventRecord(sc.done, stream));
    return VCCL_OK;
}

int launch_moe_combine_fused(MoeScratch &sc, const void *const *back, const uint64_t *capacity_rows,
                             const int32_t *const *ids, int P, int tokens, int topk, uint64_t row_bytes,
                             int num_experts, int experts_per_rank, void *const *out, hipStream_t stream) {
    const uint32_t npairs = (uint32_t)tokens * (uint32_t)topk;
    const uint32_t rv = (uint32_t)(row_bytes >> 4);
    const uint32_t tiles_per_row = (rv + 63u) / 64u;
    const uint64_t grid = (uint64_t)npairs * tiles_per_row;
    if (grid > 0x7fffffffull)
        return fail(VCCL_ERR_UNSUPPORTED, "pairs x row tiles = %llu exceeds the launch grid", (unsigned long long)grid);
    std::lock_guard<std::mutex> lk(sc.mu);
    MoePtrs ptrs;
    uint32_t *dest = nullptr;
    uint64_t *counts = nullptr, *extra = nullptr;
    // room after the counts: delta [P][P] (int64), the four layout matrices (which nobody reads
    // here), one source pointer per pair
    int rc = moe_index_phase(sc, back, ids, P, tokens, topk, num_experts, 0, nullptr, out, capacity_rows,
                             2 * ((size_t)P * P * 5 + (size_t)P * npairs), nullptr, nullptr, stream, &ptrs, &dest,
                             &counts, &extra);
    if (rc) return rc;
    int64_t *delta = reinterpret_cast<int64_t *>(extra);
    uint64_t *layout = extra + (size_t)P * P;
    const u32x4 **source = reinterpret_cast<const u32x4 **>(extra + (size_t)P * P * 5);
    moe_fused_layout_kernel<<<dim3(1), dim3(kMoeThreads), 0, stream>>>(counts, P, num_experts, experts_per_rank,
                                                                      row_bytes, ptrs.capacity_rows, layout, delta,
                                                                      nullptr);
    VCCL_HIP(hipGetLastError());
    if (npairs && rv) {
        moe_pair_source_kernel<<<dim3((npairs + kMoeThreads - 1) / kMoeThreads, P), dim3(kMoeThreads), 0, stream>>>(
            ptrs, rv, dest, npairs, experts_per_rank, delta, P, source);
        VCCL_HIP(hipGetLastError());
        RankPtrs rp;
        const FastDiv dtiles(tiles_per_row);
        const dim3 gg((uint32_t)grid, P), gb(64);
        if (rank_ptrs_inline(rp, nullptr, out, P))
            moe_combine_fused_kernel<2, true><<<gg, gb, 0, stream>>>(rp, ptrs, rv, dtiles, npairs, source);
        else
            moe_combine_fused_kernel<2, false><<<gg, gb, 0, stream>>>(rp, ptrs, rv, dtiles, npairs, source);
        VCCL_HIP(hipGetLastError());
    }
    VCCL_HIP(hipEventRecord(sc.done, stream));
    return VCCL_OK;
}

int launch_moe_unpack(MoeScratch &sc, const void *const *packed, const int32_t *const *ids, int P,
                      int tokens, int topk, uint64_t row_bytes, int num_experts, void *const *out,
                      int unpack_variant, hipStream_t stream) {
    const uint32_t npairs = (uint32_t)tokens * (uint32_t)topk;
    std::lock_guard<std::mutex> lk(sc.mu);
    MoePtrs ptrs;
    uint32_t *dest = nullptr;
    int rc = moe_index_phase(sc, packed, ids, P, tokens, topk, num_experts, 0, nullptr, out, nullptr, 0,
                             nullptr, nullptr, stream, &ptrs, &dest);
    if (rc) return rc;
    if (npairs) {
        const uint32_t rv = (uint32_t)(row_bytes >> 4);
        const uint32_t tiles = unpack_variant == 3 ? 2u : 1u;   // 1 KiB tiles per wavefront
        const uint32_t groups_per_row = (rv + 64u * tiles - 1u) / (64u * tiles);
        const uint64_t tile_grid = (uint64_t)npairs * groups_per_row;
        if (unpack_variant != 0 && tile_grid <= 0x7fffffffull && rv) {
            const dim3 g((uint32_t)tile_grid, P), b(64);
            RankPtrs rp;
            const bool inl = rank_ptrs_inline(rp, packed, out, P);
            const FastDiv dgroups(groups_per_row);
#define VCCL_UNPACK(POL, TILES)                                                                                   \
    do {                                                                                                          \
        if (inl) moe_scatter_back_tiles_kernel<POL, TILES, true><<<g, b, 0, stream>>>(rp, ptrs, rv, dgroups, dest, npairs);  \
        else moe_scatter_back_tiles_kernel<POL, TILES, false><<<g, b, 0, stream>>>(rp, ptrs, rv, dgroups, dest, npairs); \
    } while (0)
            if (unpack_variant == 3) VCCL_UNPACK(2, 2);
            else if (unpack_variant == 2) VCCL_UNPACK(2, 1);
            else VCCL_UNPACK(1, 1);
#undef VCCL_UNPACK
        } else {
            moe_scatter_back_kernel<<<dim3(npairs, P), dim3(kMoeThreads), 0, stream>>>(ptrs, rv, dest, npairs);
        }
        VCCL_HIP(hipGetLastError());
    }
    VCCL_HIP(hipEventRecord(sc.done, stream));
    return VCCL_OK;
}

}  // namespace vccl
