// Internal declarations shared by the translation units of libvccl.
// Nothing here is part of the public boundary (that is include/vccl.h).
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <condition_variable>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

#include "vccl.h"

namespace vccl {

// One contiguous piece of an exchange: `bytes` bytes from src to dst.  head is the
// number of leading bytes copied bytewise so that the vector body starts at a
// 16-byte aligned destination; lead is the number of 16-byte vectors between the
// last multiple of the tile size and that body start (tiles are cut at
// destination multiples of the tile size, the first one is short by `lead`).
struct Seg {
    const uint8_t *src;
    uint8_t *dst;
    uint64_t bytes;
    uint32_t head;
    uint32_t lead;
};
static_assert(sizeof(Seg) == 32, "descriptor layout");

// copy-engine back ends
enum { VCCL_CE_SDMA = 0, VCCL_CE_HIP_NOCU = 1, VCCL_CE_HIP_DEFAULT = 2 };
// stream ordering of the sdma back end: ready word + done word; blocking caller; ready event + done word
enum { VCCL_SYNC_MEMOPS = 0, VCCL_SYNC_HOST = 1, VCCL_SYNC_EVENT = 2 };

constexpr int kInlineSegs = 64;     // descriptors carried in the kernel arguments

struct Options {
    int cu_unroll = 1;
    int cu_wg_per_cu = 0;
    int cu_max_wg = 0;
    int cu_nontemporal = 2;
    int cu_threads = 64;
    int cu_fast_path = 1;
    int moe_gather_variant = 208;
    int moe_unpack_variant = 2;
    int p2p_close_wait_ms = 10000;   // how long vccl_p2p_close waits before it aborts the connection's transfers
    int moe_gather_full = 1;   // allow the unchecked gather kernels when pieces and slot groups are whole
    int ce_streams = 4;
    int ce_kind = 0;   // VCCL_CE_*
    int ce_max_engines = 0;
    int ce_proxy_poll = 0;   // 1: the sender proxy polls without pause while anything is in flight
    int ce_test_refuse = 0;   // test hook: bit i set = engine i refuses every copy; bit 16: every pitched copy is refused
    int ce_pitched = 1;       // equal-block AlltoAll over buffers at a constant stride: 0 plain copies, 1 pitched copies
                              // where they are expected to pay, 2 pitched copies wherever the layout allows
    int ce_sync = 0;   // VCCL_SYNC_*
    int check = 0;
    uint64_t fifo_chunk_bytes = 512u << 10;
    int fifo_slots = 8;
    int fifo_wg_per_conn = 32;
    uint64_t fifo_spin_limit = 1ull << 24;
    int fifo_scoped = 1;
};

// thread-local error message + status helper
int fail(int status, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
const char *last_error_cstr();

#define VCCL_HIP(expr)                                                                       \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess)                                                                \
            return ::vccl::fail(VCCL_ERR_HIP, "%s failed: %s (%s:%d)", #expr,                \
                                hipGetErrorString(e_), __FILE__, __LINE__);                  \
    } while (0)

// ---- descriptor staging ring (host pinned + device), one slot per in-flight launch
struct DescSlot {
    Seg *host = nullptr;
    Seg *dev = nullptr;
    hipEvent_t done = nullptr;
    bool used = false;
    bool busy = false;   // handed to a caller that has not yet recorded `done` (guarded by DescRing::mu)
};

struct DescRing {
    static constexpr int kSlots = 8;
    DescSlot slot[kSlots];
    size_t capacity = 0;   // descriptors per slot
    int next = 0;
    std::mutex mu;
    std::condition_variable cv;
    int init(size_t cap);
    void destroy();
    // Hands out the slots in turn.  Blocks while the next slot is still held by another
    // caller, and until the slot's previous launch has finished on the device.
    int acquire(DescSlot **out);
    // The caller has recorded `done` behind its launch (or has given up): the slot may go round again.
    void release(DescSlot *s);
};

// ---- CU copy path
struct CopyPlan {
    std::vector<Seg> segs;       // non-empty descriptors, tile_begin / head filled in
    uint64_t total_tiles = 0;
    uint32_t max_tiles = 0;      // tiles of the longest descriptor (grid x)
    bool all_aligned = false;    // every descriptor: 16-byte aligned ends, whole vectors
    bool fast = false;           // tiled for (and to be run by) the all-aligned kernel
    int threads = 64;            // lanes per workgroup the tiles were sized for
    uint64_t bytes = 0;
};
// Fills tile_begin/head for plan.segs (src, dst, bytes already set).
// Tiles are unroll * threads vectors; allow_fast lets an all-aligned plan select the
// kernel without head / tail / realignment code (it needs the full grid).
int plan_tiles(CopyPlan &plan, int unroll, int threads, bool allow_fast);
int launch_copy(const CopyPlan &plan, const Options &opt, int cu_count, DescRing &ring,
                hipStream_t stream);

// Equal-block AlltoAll whose descriptors are derived in the kernel from the rank
// pointers (no table, no upload); applies when everything is 16-byte aligned.
bool uniform_alltoall_applies(void *const *sendbuf, void *const *recvbuf, uint64_t bytes_per_peer, int P,
                              const Options &opt);
int launch_uniform_alltoall(void *const *sendbuf, void *const *recvbuf, uint64_t bytes_per_peer, int P,
                            const Options &opt, hipStream_t stream);

// ---- staged FIFO SendRecv (CU_STAGED)
struct FifoState {
    uint8_t *slots = nullptr;        // connections x fifo_slots x chunk bytes
    uint64_t *counters = nullptr;    // per (connection, lane-group): head, tail
    uint32_t *status = nullptr;      // device words: [0] non-zero while the running operation has given up,
                                     // [1] number of operations that gave up since the allocation
    uint32_t *errors_host = nullptr; // pinned word the status query copies [1] into
    uint32_t errors_reported = 0;
    struct FifoConn *conns_dev = nullptr;   // table for operations with more connections than fit
    struct FifoConn *conns_host = nullptr;  // the kernel arguments (pinned staging)
    hipEvent_t done = nullptr;       // recorded behind the last staged operation
    hipStream_t last_stream = nullptr;
    size_t slots_bytes = 0;
    size_t counters_n = 0;
    size_t conns_n = 0;
    void destroy();
};
// Staged operations that are in flight together (different streams) each need FIFO
// memory of their own, as every connection of a kernel-driven library has; a call takes
// an idle state if there is one and otherwise queues behind the oldest.
struct FifoPool {
    static constexpr int kStates = 8;
    FifoState st[kStates];
    unsigned next = 0;
    std::mutex mu;
    void destroy();
};
struct FifoConn {
    const uint8_t *src;
    uint8_t *dst;
    uint64_t bytes;
};
// Waits for the last staged operation and reports whether a bounded wait gave up.
int fifo_last_status(FifoPool &pool, uint32_t *out);
int launch_fifo(FifoPool &pool, const std::vector<FifoConn> &conns, const Options &opt,
                int cu_count, hipStream_t stream);

// ---- MoE pack
struct MoeScratch {
    uint32_t *hist = nullptr;    // [P][blocks][E] per-block histograms, then offsets
    size_t hist_n = 0;
    void **ptrs = nullptr;       // device copies of the x / ids / packed pointer arrays
    void **ptrs_host = nullptr;  // pinned staging for them
    hipEvent_t done = nullptr;
    size_t ptrs_n = 0;
    std::mutex mu;
    void destroy();
};
// experts_per_rank == 0: one row per (token, slot), sorted by expert id.  experts_per_rank > 0:
// one row per (token, destination rank), counts per rank, optional slot-to-row maps.
int launch_moe_pack(MoeScratch &sc, const void *const *x, const int32_t *const *ids, int P,
                    int tokens, int topk, uint64_t row_bytes, int num_experts, int experts_per_rank,
                    void *const *packed, uint64_t *counts_dev, uint64_t *counts_host,
                    uint32_t *const *slot_row, uint32_t *bad_ids_dev, int gather_variant, int gather_full,
                    hipStream_t stream);

// The pack for callers that cannot allocate: index data in a file-scope device array
// whose address moe_static_scratch_init asks for once per device (that device current).
int moe_static_scratch_init(int device);
int launch_moe_pack_noalloc(int device, const void *const *x, const int32_t *const *ids, int P, int tokens,
                            int topk, uint64_t row_bytes, int num_experts, void *const *packed,
                            uint64_t *counts_dev, uint32_t *bad_ids_dev, int gather_variant, int gather_full,
                            hipStream_t stream);

// Pack and exchange in one pass: rows go from x[s] straight into recv[r] where the
// exchange after a pack would have put them.
int launch_moe_dispatch_fused(MoeScratch &sc, const void *const *x, const int32_t *const *ids, int P,
                              int tokens, int topk, uint64_t row_bytes, int num_experts,
                              int experts_per_rank, void *const *recv, const uint64_t *capacity_rows,
                              uint64_t *counts_dev, uint64_t *layout_dev, uint64_t *layout_host,
                              uint32_t *status_dev, int gather_full, hipStream_t stream);

// The way back in one pass: row t*K+k of out[s] is read straight from back[r].
int launch_moe_combine_fused(MoeScratch &sc, const void *const *back, const uint64_t *capacity_rows,
                             const int32_t *const *ids, int P, int tokens, int topk, uint64_t row_bytes,
                             int num_experts, int experts_per_rank, void *const *out, hipStream_t stream);

int launch_moe_unpack(MoeScratch &sc, const void *const *packed, const int32_t *const *ids, int P,
                      int tokens, int topk, uint64_t row_bytes, int num_experts, void *const *out,
                      int unpack_variant, hipStream_t stream);

// ---- co-run probe
int launch_fma_probe(float *out, uint64_t *clocks, uint32_t workgroups, uint32_t threads, uint64_t iters,
                     hipStream_t stream);

// kind: 0 read-only (dst = 64-byte sink), 1 write-only, 2 copy, 3 write rows of row_bytes at row_index[i]
int launch_hbm_probe(int kind, const void *src, void *dst, uint64_t bytes, int threads, int vecs,
                     const uint32_t *row_index, uint64_t n_rows, uint64_t row_bytes, hipStream_t stream);

// ---- copy-engine proxy
struct CeCopy {
    const void *src;
    void *dst;
    uint64_t bytes;
    int receiver;  // >= 0: SendRecv copy whose destination is read from that rank's handshake record
};
// `rows` blocks of `width` bytes, row i at src + i * src_pitch going to dst + i * dst_pitch:
// one pitched engine copy (what the blocks of one rank are in an equal-block AlltoAll whose
// buffers on the other side lie at a constant stride).
struct CeRect {
    const void *src;
    void *dst;
    uint64_t width, rows, src_pitch, dst_pitch;
};
// The receiver-owned handshake record of a connection between two PROCESSES (Section
// 3.2: P2pRegInfo in host shared memory, mapped into the sender at connect).  The
// paper's 1-bit flags are sequence numbers that only grow: transfer n of the connection
// is ready / started / done once the field has reached n.
struct P2pShared {
    uint64_t magic;                      // written last by the exporting process
    uint64_t capacity;                   // bytes of the registered receive buffer
    uint64_t alloc_offset;               // where that buffer starts inside the exported allocation
    uint8_t ipc_handle[64];              // hipIpcMemHandle_t of the allocation
    std::atomic<uint64_t> receiverRegOffset;   // receiverRegAddr: offset of transfer n inside the registered buffer,
    std::atomic<uint64_t> receiverRegBytes;    // and how many bytes the receiver expects (published before ready)
    std::atomic<uint64_t> receiverReady;
    std::atomic<uint64_t> copyStarted;
    std::atomic<uint64_t> copyDone;
    std::atomic<uint64_t> mismatches;    // transfers whose byte counts disagreed (nothing was copied for them)
    std::atomic<uint32_t> sender_attached;
    std::atomic<uint32_t> receiver_closed;
    std::atomic<uint32_t> aborted;       // either side gave up: every outstanding and later transfer fails
    int32_t receiver_pid;
};
static_assert(std::atomic<uint64_t>::is_always_lock_free, "the record is shared between processes");
constexpr uint64_t kP2pMagic = 0x5643434c50325031ull;   // "VCCLP2P1"

class Proxy;
Proxy *proxy_create(int device, int max_streams);
// One side of a transfer over a cross-process connection, ordered on `stream` like any
// other copy-engine operation.  role 1 (sender): copy `bytes` from src into the mapped
// receive buffer once the record shows transfer `seq` ready.  role 2 (receiver): when the
// stream has reached the operation and transfer seq - 1 has started, publish (offset,
// bytes) and raise ready; the stream resumes when the record shows transfer seq done.
int proxy_submit_remote(Proxy *p, int role, P2pShared *sh, uint8_t *mapped_buffer, uint64_t seq, const void *src,
                        uint64_t offset, uint64_t bytes, const Options &opt, hipStream_t stream);
void proxy_destroy(Proxy *p);
// Orders the copies after everything already on `stream`, has the proxy thread
// issue them on the internal copy streams, and makes `stream` wait for them.
// `receivers` (may be null) lists (receiving rank, application buffer) pairs that
// go through the per-connection handshake record.
int proxy_submit(Proxy *p, std::vector<CeCopy> &&copies, const Options &opt, hipStream_t stream,
                 const std::vector<std::pair<int, void *>> *receivers, std::vector<CeRect> *rects = nullptr);
// Whether P pitched copies of P blocks of `block_bytes` are expected to finish before the
// P * P plain copies they replace (sdma back end).
bool proxy_pitched_pays(int P, uint64_t block_bytes);
int proxy_reginfo(Proxy *p, int receiver, uint64_t *ready, uint64_t *started, uint64_t *done,
                  void **addr);
int proxy_drain(Proxy *p);
bool proxy_drain_for(Proxy *p, double seconds);   // false if operations were still in flight at the deadline
// Whether the HSA/SDMA back end came up on this device (and, if not, why).
bool proxy_sdma_available(Proxy *p, const char **why);
int proxy_engine_count(Proxy *p);
uint64_t proxy_sdma_errors(Proxy *p);
uint64_t proxy_refused_pieces(Proxy *p);
uint64_t proxy_pitched_copies(Proxy *p);
void proxy_set_always_poll(Proxy *p, bool on);
vccl_monitor *proxy_monitor(Proxy *p, int primitive);
void proxy_stats(Proxy *p, uint64_t *ops, uint64_t *copies, uint64_t *bytes, uint64_t *issue_ns);
int proxy_cpu_time(Proxy *p, uint64_t *sender_ns, uint64_t *receiver_ns);
uint64_t proxy_engine_bytes(Proxy *p, int engine);

}  // namespace vccl
