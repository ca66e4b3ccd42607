// Staged SendRecv on compute units: the two-step intra-node pattern of a
// kernel-driven library (paper Section 2.2): sender workgroups copy the
// application buffer chunk by chunk into a chunk FIFO, receiver workgroups copy
// each chunk out into the destination as it arrives.  It exists as the baseline
// the zero-copy and copy-engine paths are compared with; it moves every byte
// twice and holds compute units for the whole transfer.
//
// Each connection is served by W independent sender/receiver workgroup pairs.
// Pair j owns slice j of every chunk and its own head/tail counters, so every
// counter has exactly one writer and one reader.  Chunk k lives in slot
// k mod slots; the sender waits while head - tail == slots, the receiver while
// tail == head.  Every wait is bounded: after spin_limit polls the workgroup
// raises the status word and leaves, so the grid always drains.
//
// Two ways of making a chunk visible to the receiver.  Fenced: plain stores, then a
// device-scope release on the counter (a write-back of the XCD's L2) and an acquire on
// the receiver's poll (an invalidate); those cache operations serialise per XCD and
// were the whole cost of a chunk (about 0.7 us each, 8 to 32 of them per chunk time).
// Scoped (default): the slot bytes themselves are stored and loaded at device scope,
// the sender waits for its stores to be acknowledged, and the counters move relaxed.
#include "common.h"

namespace vccl {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kFifoThreads = 256;
constexpr int kFifoInlineConns = 64;   // connections that travel in the kernel arguments

struct FifoArgs {
    const FifoConn *conns;   // device array, or null: the connections are in `inl`
    FifoConn inl[kFifoInlineConns];
    uint8_t *slots;          // [conn][slot][chunk_bytes]
    uint64_t *counters;      // [conn][W][2]: head, tail
    uint32_t *status;        // [0] this operation gave up, [1] operations that gave up so far
    uint64_t chunk_bytes;
    uint64_t spin_limit;
    uint32_t nslots;
    uint32_t W;
};

__global__ void fifo_zero_words_kernel(uint32_t *words, uint32_t n) {
    if (threadIdx.x < n) words[threadIdx.x] = 0;
}

__global__ void fifo_reset_kernel(uint64_t *counters, uint32_t n, uint32_t *status) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) counters[i] = 0;
    if (i == 0) status[0] = 0;
}

// Copy [a, b) of a chunk; `from`/`to` are the chunk bases.  Vector path when both
// sides are 16-byte aligned at `a`, bytewise otherwise.
__device__ __forceinline__ void copy_range(const uint8_t *from, uint8_t *to, uint64_t a, uint64_t b) {
    const uint8_t *s = from + a;
    uint8_t *d = to + a;
    const uint64_t n = b - a;
    if (((reinterpret_cast<uintptr_t>(s) | reinterpret_cast<uintptr_t>(d)) & 15u) == 0) {
        const uint64_t nv = n >> 4;
        const u32x4 *sv = reinterpret_cast<const u32x4 *>(s);
        u32x4 *dv = reinterpret_cast<u32x4 *>(d);
        // Streaming stores: the data is not read again by this workgroup, and little
        // dirty data in L2 keeps the write-back of the release cheap.
        for (uint64_t i = threadIdx.x; i < nv; i += 8 * kFifoThreads) {
            u32x4 r[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (i + u * kFifoThreads < nv) r[u] = sv[i + u * kFifoThreads];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (i + u * kFifoThreads < nv) __builtin_nontemporal_store(r[u], dv + i + u * kFifoThreads);
        }
        for (uint64_t t = (nv << 4) + threadIdx.x; t < n; t += kFifoThreads) d[t] = s[t];
    } else {
        for (uint64_t t = threadIdx.x; t < n; t += kFifoThreads) d[t] = s[t];
    }
}

// FIFO memory seen through device-scope (sc1) accesses only: such a store is written
// through to memory before it is acknowledged and such a load never takes a line another
// XCD's cache may hold stale, so a sender that has waited for its stores and a receiver
// that reads with these loads need no cache write-back or invalidate around the
// counters - the same way the counters themselves travel.  The descriptor sits on a
// wave-uniform base; offsets stay below 2 GiB (a chunk is at most 64 MiB).
struct SlotView {
    __amdgpu_buffer_rsrc_t rsrc;
    __device__ __forceinline__ explicit SlotView(const uint8_t *base) {
        rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, 0x7fffffff, 0x00020000 /* raw dwords */);
    }
    __device__ __forceinline__ u32x4 load16(uint32_t off) const {
        return __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 16 /* sc1 */);
    }
    __device__ __forceinline__ void store16(uint32_t off, u32x4 v) const {
        __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, off, 0, 16 /* sc1 */);
    }
    __device__ __forceinline__ uint8_t load8(uint32_t off) const {
        return __builtin_amdgcn_raw_buffer_load_b8(rsrc, off, 0, 16 /* sc1 */);
    }
    __device__ __forceinline__ void store8(uint32_t off, uint8_t v) const {
        __builtin_amdgcn_raw_buffer_store_b8(v, rsrc, off, 0, 16 /* sc1 */);
    }
};

// copy_range with the FIFO side of the copy going through a SlotView.  SIDE 0: memory
// to slot (sender), SIDE 1: slot to memory (receiver).
template <int SIDE>
__device__ __forceinline__ void copy_range_scoped(const uint8_t *from, uint8_t *to, uint64_t a, uint64_t b) {
    const uint8_t *s = from + a;
    uint8_t *d = to + a;
    const uint32_t n = (uint32_t)(b - a);
    const SlotView slot(SIDE == 0 ? d : s);
    if (((reinterpret_cast<uintptr_t>(s) | reinterpret_cast<uintptr_t>(d)) & 15u) == 0) {
        const uint32_t nv = n >> 4;
        const u32x4 *sv = reinterpret_cast<const u32x4 *>(s);
        u32x4 *dv = reinterpret_cast<u32x4 *>(d);
        // rounds of up to 8 vectors per lane: all loads of a round are in flight together
        for (uint32_t i = threadIdx.x; i < nv; i += 8 * kFifoThreads) {
            u32x4 r[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint32_t j = i + u * kFifoThreads;
                if (j < nv) r[u] = SIDE == 0 ? __builtin_nontemporal_load(sv + j) : slot.load16(j * 16u);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint32_t j = i + u * kFifoThreads;
                if (j < nv) {
                    if (SIDE == 0) slot.store16(j * 16u, r[u]);
                    else __builtin_nontemporal_store(r[u], dv + j);
                }
            }
        }
        for (uint32_t t = (nv << 4) + threadIdx.x; t < n; t += kFifoThreads) {
            if (SIDE == 0) slot.store8(t, s[t]);
            else d[t] = slot.load8(t);
        }
    } else {
        for (uint32_t t = threadIdx.x; t < n; t += kFifoThreads) {
            if (SIDE == 0) slot.store8(t, s[t]);
            else d[t] = slot.load8(t);
        }
    }
}

// SCOPED: the FIFO is reached through SlotView and the counters move with relaxed
// device-scope accesses; otherwise plain accesses ordered by a release on the
// sender's counter store and an acquire on the receiver's poll.
template <bool SCOPED>
__global__ __launch_bounds__(kFifoThreads) void fifo_sendrecv_kernel(FifoArgs a) {
    __shared__ int give_up;
    // sender and receiver of a pair sit next to each other in the launch order
    const uint32_t side = blockIdx.x & 1u;
    const uint32_t pair = blockIdx.x >> 1;
    const uint32_t conn = pair / a.W, j = pair - conn * a.W;
    const FifoConn c = a.conns ? a.conns[conn] : a.inl[conn];
    uint64_t *head = a.counters + ((size_t)conn * a.W + j) * 2;
    uint64_t *tail = head + 1;
    uint8_t *fifo = a.slots + (size_t)conn * a.nslots * a.chunk_bytes;
    const uint64_t nchunks = (c.bytes + a.chunk_bytes - 1) / a.chunk_bytes;
    // slice j of a chunk, on 16-byte boundaries of the chunk
    const uint64_t cv = a.chunk_bytes >> 4;
    const uint64_t lo = (cv * j / a.W) << 4, hi = (cv * (j + 1) / a.W) << 4;
    if (threadIdx.x == 0) give_up = 0;
    __syncthreads();
    uint64_t seen = 0;   // lane 0: the other side's counter as last read
    for (uint64_t k = 0; k < nchunks; ++k) {
        const uint64_t off = k * a.chunk_bytes;
        const uint64_t len = min(a.chunk_bytes, c.bytes - off);
        const uint64_t b0 = min(lo, len), b1 = min(hi, len);
        uint8_t *slot = fifo + (k % a.nslots) * a.chunk_bytes;
        if (threadIdx.x == 0) {
            uint64_t polls = 0;
            if (side == 0) {
                // Slot reuse carries no data back to the sender: a relaxed read is enough,
                // and none is needed while the last value seen still leaves a slot free.
                while (k - seen >= a.nslots) {
                    seen = __hip_atomic_load(tail, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (k - seen < a.nslots) break;
                    if (++polls > a.spin_limit || __hip_atomic_load(a.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
                        give_up = 1;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
            } else {
                // Fenced protocol: the acquire invalidates this compute unit's view of the
                // slots before they are read.  Chunks below the value seen were complete
                // when it was read, and a slot cannot be refilled (and so go stale here)
                // before a later poll has seen the refill.
                while (seen <= k) {
                    seen = SCOPED ? __hip_atomic_load(head, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                  : __hip_atomic_load(head, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
                    if (seen > k) break;
                    if (++polls > a.spin_limit || __hip_atomic_load(a.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
                        give_up = 1;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
            }
        }
        __syncthreads();
        if (give_up) {
            // the first workgroup to give up counts the operation as failed
            if (threadIdx.x == 0 &&
                __hip_atomic_exchange(a.status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u)
                __hip_atomic_fetch_add(a.status + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        if (SCOPED) {
            if (side == 0) copy_range_scoped<0>(c.src + off, slot, b0, b1);
            else copy_range_scoped<1>(slot, c.dst + off, b0, b1);
        } else {
            if (side == 0) copy_range(c.src + off, slot, b0, b1);
            else copy_range(slot, c.dst + off, b0, b1);
        }
        // Every lane waits for its own loads and stores to finish, the workgroup meets,
        // then one lane moves the counter.  Scoped: the sender's stores were written
        // through before they were acknowledged, so a relaxed counter store is enough.
        // Fenced: the sender's release writes the slot data back so that a receiver on
        // another XCD sees it.  The receiver only has to have finished reading the slot,
        // so its counter store is relaxed either way.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (threadIdx.x == 0) {
            if (side == 0 && !SCOPED) __hip_atomic_store(head, k + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
            else __hip_atomic_store(side == 0 ? head : tail, k + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

void FifoState::destroy() {
    if (done) {
        (void)hipEventSynchronize(done);
        (void)hipEventDestroy(done);
        done = nullptr;
    }
    if (slots) (void)hipFree(slots);
    if (counters) (void)hipFree(counters);
    if (status) (void)hipFree(status);
    if (errors_host) (void)hipHostFree(errors_host);
    if (conns_dev) (void)hipFree(conns_dev);
    if (conns_host) (void)hipHostFree(conns_host);
    slots = nullptr;
    counters = nullptr;
    status = nullptr;
    errors_host = nullptr;
    conns_dev = nullptr;
    conns_host = nullptr;
    slots_bytes = counters_n = conns_n = 0;
    errors_reported = 0;
    last_stream = nullptr;
}

void FifoPool::destroy() {
    std::lock_guard<std::mutex> lk(mu);
    for (FifoState &s : st) s.destroy();
}

// Nothing here makes the calling thread wait for the device in the common case: a
// staged operation is ordered behind the previous one (which owns the FIFO memory)
// by an event the stream waits on, up to 64 connections travel in the kernel
// arguments, and whether a wait gave up is counted on the device and read only when
// the status is asked for.  The thread does wait when the FIFO has to grow or when an
// operation has more connections than the kernel arguments hold.
int launch_fifo(FifoPool &pool, const std::vector<FifoConn> &conns, const Options &opt, int cu_count,
                hipStream_t stream) {
    const size_t nconn = conns.size();
    // Both sides of every pair must be able to be resident together; keep the grid
    // well inside what the device holds at once.
    uint32_t W = (uint32_t)opt.fifo_wg_per_conn;
    const uint64_t max_wg = (uint64_t)cu_count * 2;
    while (W > 1 && 2ull * W * nconn > max_wg) W >>= 1;
    if (2ull * W * nconn > (uint64_t)cu_count * 8)
        return fail(VCCL_ERR_UNSUPPORTED, "%zu connections need more co-resident workgroups than the device holds",
                    nconn);
    const uint64_t cv = opt.fifo_chunk_bytes >> 4;
    if (cv < W) W = (uint32_t)cv;
    const size_t slots_bytes = nconn * (size_t)opt.fifo_slots * opt.fifo_chunk_bytes;
    const size_t counters_n = nconn * W * 2;

    std::lock_guard<std::mutex> lk(pool.mu);
    // The state this stream used last (its operations follow each other anyway), else an
    // idle one (never used, or its last operation has finished), else the oldest.
    FifoState *pick = nullptr;
    for (FifoState &cand : pool.st)
        if (cand.done && cand.last_stream == stream) pick = &cand;
    for (int i = 0; i < FifoPool::kStates && !pick; ++i)
        if (!pool.st[i].done || hipEventQuery(pool.st[i].done) == hipSuccess) pick = &pool.st[i];
    if (!pick) {
        pick = &pool.st[pool.next];
        pool.next = (pool.next + 1) % FifoPool::kStates;
    }
    pick->last_stream = stream;
    FifoState &st = *pick;
    if (!st.done) {
        VCCL_HIP(hipEventCreateWithFlags(&st.done, hipEventDisableTiming));
        VCCL_HIP(hipEventRecord(st.done, stream));
    }
    if (!st.status) {
        VCCL_HIP(hipMalloc((void **)&st.status, 2 * sizeof(uint32_t)));
        fifo_zero_words_kernel<<<dim3(1), dim3(64), 0, stream>>>(st.status, 2);   // ordered before the first use
        VCCL_HIP(hipGetLastError());
        VCCL_HIP(hipHostMalloc((void **)&st.errors_host, sizeof(uint32_t), hipHostMallocDefault));
        *st.errors_host = 0;
    }
    const bool table = nconn > (size_t)kFifoInlineConns;
    if (slots_bytes > st.slots_bytes || counters_n > st.counters_n || table)
        VCCL_HIP(hipEventSynchronize(st.done));   // memory still in use is about to be replaced
    if (slots_bytes > st.slots_bytes) {   // the FIFO is allocated on first use and grown on demand
        if (st.slots) VCCL_HIP(hipFree(st.slots));
        st.slots = nullptr;
        st.slots_bytes = 0;
        VCCL_HIP(hipMalloc((void **)&st.slots, slots_bytes));
        st.slots_bytes = slots_bytes;
    }
    if (counters_n > st.counters_n) {
        if (st.counters) VCCL_HIP(hipFree(st.counters));
        st.counters = nullptr;
        st.counters_n = 0;
        VCCL_HIP(hipMalloc((void **)&st.counters, counters_n * sizeof(uint64_t)));
        st.counters_n = counters_n;
    }
    FifoArgs a;
    a.conns = nullptr;
    if (table) {
        if (nconn > st.conns_n) {
            if (st.conns_dev) VCCL_HIP(hipFree(st.conns_dev));
            if (st.conns_host) VCCL_HIP(hipHostFree(st.conns_host));
            st.conns_dev = nullptr;
            st.conns_host = nullptr;
            st.conns_n = 0;
            VCCL_HIP(hipMalloc((void **)&st.conns_dev, nconn * sizeof(FifoConn)));
            VCCL_HIP(hipHostMalloc((void **)&st.conns_host, nconn * sizeof(FifoConn), hipHostMallocDefault));
            st.conns_n = nconn;
        }
        for (size_t i = 0; i < nconn; ++i) st.conns_host[i] = conns[i];
        VCCL_HIP(hipMemcpyAsync(st.conns_dev, st.conns_host, nconn * sizeof(FifoConn), hipMemcpyHostToDevice,
                                stream));
        a.conns = st.conns_dev;
    } else {
        for (size_t i = 0; i < nconn; ++i) a.inl[i] = conns[i];
    }
    // One staged operation at a time owns this state's FIFO memory, whatever stream it is on.
    VCCL_HIP(hipStreamWaitEvent(stream, st.done, 0));
    fifo_reset_kernel<<<dim3((uint32_t)((counters_n + 255) / 256)), dim3(256), 0, stream>>>(
        st.counters, (uint32_t)counters_n, st.status);
    VCCL_HIP(hipGetLastError());
    a.slots = st.slots;
    a.counters = st.counters;
    a.status = st.status;
    a.chunk_bytes = opt.fifo_chunk_bytes;
    a.spin_limit = opt.fifo_spin_limit;
    a.nslots = (uint32_t)opt.fifo_slots;
    a.W = W;
    if (opt.fifo_scoped)
        fifo_sendrecv_kernel<true><<<dim3((uint32_t)(2 * W * nconn)), dim3(kFifoThreads), 0, stream>>>(a);
    else
        fifo_sendrecv_kernel<false><<<dim3((uint32_t)(2 * W * nconn)), dim3(kFifoThreads), 0, stream>>>(a);
    VCCL_HIP(hipGetLastError());
    VCCL_HIP(hipEventRecord(st.done, stream));
    return VCCL_OK;
}

// Waits for the staged operations issued so far; *out is non-zero when one of them,
// since the last time this was asked, ran out of polls.
int fifo_last_status(FifoPool &pool, uint32_t *out) {
    std::lock_guard<std::mutex> lk(pool.mu);
    *out = 0;
    for (FifoState &st : pool.st) {
        if (!st.done || !st.status) continue;
        VCCL_HIP(hipEventSynchronize(st.done));
        VCCL_HIP(hipMemcpy(st.errors_host, st.status + 1, sizeof(uint32_t), hipMemcpyDeviceToHost));
        const uint32_t now = *st.errors_host;
        if (now != st.errors_reported) *out = 1u;
        st.errors_reported = now;
    }
    return VCCL_OK;
}

}  // namespace vccl
