// Copy-engine path: a host proxy thread moves the data with the GPU's SDMA copy
// engines so that no kernel is launched for the transfer and no compute unit is
// touched (the paper's SM-free P2P: data movement by copy engines, control on a
// CPU proxy thread with completion found by polling, Section 3.2 items 1-2).
//
// Two back ends:
//
//  "sdma" (default)  The proxy submits every copy straight to an SDMA engine
//      through the HSA runtime, each piece to the engine with the fewest bytes so
//      far.  Stream order is kept the way the paper ends up doing it (Section 3.2
//      item 3): the caller's stream tells the proxy when the preceding work is done
//      (the paper's proxyReadyEvent) - by an event the proxy polls (ordering
//      "event") or by WRITING a sequence number into a host-visible ready word
//      (ordering "memops") - the proxy issues the copies, polls their completion
//      signal, and then stores the sequence number into a signal word the caller's
//      stream WAITS on (the role of proxyOpCount returning to zero).  No kernel of
//      this library, no host callback, and the calling thread never blocks; whether
//      the HIP runtime needs a helper kernel for its stream operations is its
//      business (the wait needs none when the command processor carries it out).
//      Ordering "host" uses no stream operation at all: the caller blocks.
//
//  "hip_nocu" / "hip_default"  hipMemcpyAsync on internal streams, ordered with
//      events (record `ready`, internal streams wait, record `done[i]`, caller's
//      stream waits).  Whether hipMemcpyDeviceToDeviceNoCU really avoids compute
//      units depends on the HIP runtime that is loaded, so this is not the default.
//
// The proxy polls only where polling buys latency (right after something moved,
// and around the time a pending operation is due, going by what operations of the
// same shape took before); in between it sleeps, so a transfer costs a fraction of
// its length in processor time (Section 4.1 charges the SM-free design about 2 % of
// host CPU).  Option ce_proxy_poll = 1 makes it poll without pause, as in the paper.
//
// hipLaunchHostFunc is never used: host callbacks of independent streams may be
// serialised, which is the deadlock the paper describes.
//
// For SendRecv each connection also walks the receiver-owned handshake record of
// Section 3.2 (receiverRegAddr / receiverReady -> copyStarted -> copyDone), with
// the two roles on two threads as in the paper: a receiver proxy publishes the
// application buffer and raises ready once the previous transfer on the connection
// has started; the sender proxy (the thread that drives the copy engines) issues
// the copies of a transfer only when its connection shows ready, reads the
// destination from the record, and marks started / done.  The paper's 1-bit flags
// are kept here as monotonically increasing sequence numbers, which need no reset
// between operations; the calling thread only draws the numbers and never waits.
// Between two PROCESSES the same record lives in shared memory (P2pShared): either
// side of such a transfer is an operation of its process's proxy like any other.
#include <hsa/hsa.h>
#include <hsa/hsa_ext_amd.h>

#include <pthread.h>
#include <sys/prctl.h>
#include <time.h>

#include <chrono>
#include <condition_variable>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <thread>
#include <unordered_map>

#include "common.h"

namespace vccl {

namespace {
constexpr int kMaxStreams = 8;
constexpr int kMaxEngines = 16;
constexpr uint64_t kMinPiece = 1u << 20;   // copies are cut no finer than this
constexpr uint64_t kMaxPiece = 16u << 20;  // and a piece is no longer than this (engines reach their rate from there)

struct RegInfo {  // one per receiving rank
    std::atomic<void *> receiverRegAddr{nullptr};
    std::atomic<uint64_t> receiverReady{0};
    std::atomic<uint64_t> copyStarted{0};
    std::atomic<uint64_t> copyDone{0};
    uint64_t drawn = 0;   // last sequence number handed to a transfer (guarded by handshake_mu)
};

struct RecvPost {   // what the receiver proxy publishes for one transfer on one connection
    int rank;
    uint64_t seq;
    void *addr;
};

struct Op {
    std::vector<CeCopy> copies;
    std::vector<CeRect> rects;                    // pitched copies (sdma back end only)
    std::vector<std::pair<int, uint64_t>> conns;  // (receiver rank, sequence number)
    int kind = VCCL_CE_SDMA;
    // event back end
    hipEvent_t ready = nullptr;
    hipEvent_t done[kMaxStreams] = {};
    int nstreams = 0;
    int want_streams = 1;
    int state = 0;             // 0 queued, 1 issued, 2 failed   (guarded by Proxy::mu)
    hipError_t err = hipSuccess;
    int refs = 0;              // caller + proxy                 (guarded by Proxy::mu)
    // sdma back end
    volatile uint64_t *ready_word = nullptr;   // pinned host memory, written by the caller's stream
    uint64_t *done_word = nullptr;             // signal memory, waited on by the caller's stream
    hsa_signal_t left = {0};                   // outstanding copies
    uint64_t seq = 0;
    int primitive = 1;                         // 0 SendRecv, 1 AlltoAll(v): which monitor sees the op
    uint64_t monitor_id = 0;
    bool host_sync = false;                    // no stream memory operations: the caller blocks
    bool ready_event = false;                  // readiness is found by polling the `ready` event, not the ready word
    int max_engines = 0;
    uint32_t refuse_mask = 0;                  // test hook: engines (by index) treated as refusing every copy
    bool sdma_failed = false;
    uint64_t bytes = 0;                        // bytes handed to the engines
    uint64_t t_issue_ns = 0;                   // when they were handed over
    uint64_t est_ns = 0;                       // how long the engines are expected to take
    uint64_t shape = 0;                        // key of the operation's shape in the proxy's history
    uint64_t t_seen_busy_ns = 0;               // the last poll that found it incomplete
    // one side of a transfer over a cross-process connection (0 = none, 1 = sender, 2 = receiver)
    int remote_role = 0;
    P2pShared *remote = nullptr;
    uint8_t *remote_buffer = nullptr;          // sender: the receiver's registered buffer as mapped here
    uint64_t remote_seq = 0, remote_offset = 0, remote_bytes = 0;
};
}  // namespace

class Proxy {
public:
    int device = 0;
    int max_streams = kMaxStreams;
    hipStream_t streams[kMaxStreams] = {};
    std::thread th, receiver_th;
    std::mutex mu, handshake_mu, recv_mu;
    std::condition_variable cv_work, cv_issued, cv_idle, cv_recv;
    std::deque<Op *> queue;
    std::deque<RecvPost> recv_queue;   // in the order the numbers were drawn (guarded by recv_mu)
    bool recv_stop = false;
    std::vector<Op *> waiting;   // sdma ops whose ready word has not arrived (proxy thread only)
    std::vector<Op *> pending;   // issued, completion not yet observed   (proxy thread only)
    std::vector<Op *> free_ops;
    bool stop = false;
    size_t in_flight = 0;        // queued + waiting + pending
    RegInfo reg[VCCL_MAX_RANKS];
    std::atomic<uint64_t> n_ops{0}, n_copies{0}, n_bytes{0}, issue_ns{0}, sdma_errors{0}, n_refused{0}, n_pitched{0};
    std::atomic<uint64_t> engine_bytes[kMaxEngines] = {};   // bytes handed to each engine so far
    // sdma back end
    bool sdma_ok = false;
    std::string sdma_why;
    hsa_agent_t agent = {0};
    bool hsa_up = false;
    uint32_t engine_bit[kMaxEngines] = {};
    int nengines = 0;
    unsigned next_engine = 0;
    void *warm = nullptr;
    // one window monitor per primitive over the operations issued (Section 3.4)
    vccl_monitor *monitor[2] = {nullptr, nullptr};
    uint64_t next_monitor_id = 0;
    static uint64_t now_ns() {
        return (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(
                   std::chrono::steady_clock::now().time_since_epoch()).count();
    }

    // How long an operation is expected to take; the sender proxy sleeps on this before it
    // starts polling.  Collectives repeat: the estimate for a shape (bytes to within 1/16,
    // number of pieces, engines in use) is what operations of that shape took before, kept in `history`.
    // A shape seen for the first time takes a model of the engines: they work in parallel,
    // each through its own pieces at kEngineRate with kCopyCost of fixed time per piece, and
    // all together no faster than kAllRate and one piece per kAllCopyCost.  The constants
    // lean towards too short an estimate: that costs some polling, too long a one costs latency.
    static constexpr double kEngineRate = 60.0;    // bytes copied per nanosecond (= GB/s), one engine alone
    static constexpr double kAllRate = 760.0;      // bytes copied per nanosecond, all engines together
    static constexpr double kCopyCost = 6500.0;    // nanoseconds per piece on its engine
    static constexpr double kAllCopyCost = 980.0;  // nanoseconds per piece over all engines (about a million copies a second)
    // Pitched copies have no engine argument; the runtime runs them one after another on one
    // engine, each in about kRectCost plus its bytes at kRectRate.
    static constexpr double kRectCost = 11000.0;   // nanoseconds per pitched copy
    static constexpr double kRectRate = 60.0;      // bytes per nanosecond inside a pitched copy
    std::unordered_map<uint64_t, uint64_t> history;   // shape -> nanoseconds (proxy thread only)
    static uint64_t shape_key(uint64_t bytes, size_t pieces, int engines) {
        int top = 63 - __builtin_clzll(bytes | 1);
        const uint64_t coarse = top > 4 ? (bytes >> (top - 4)) << (top - 4) : bytes;
        return (coarse * 0x9E3779B97F4A7C15ull ^ (uint64_t)pieces) + (uint64_t)engines;
    }
    void learn(const Op *op, uint64_t t_done);
    std::atomic<bool> always_poll{false};          // option "ce_proxy_poll": never sleep while something is in flight
    std::mutex started_mu;
    std::condition_variable cv_started;   // copyStarted of some connection has advanced
    uint64_t nap_ns(uint64_t now, uint64_t last_progress) const;
    void mark_started(Op *op);
    void run();
    void run_receiver();
    bool receivers_ready(const Op *op) const;
    void issue_events(Op *op);
    bool issue_sdma(Op *op);
    bool issue_remote_recv(Op *op);
    bool stream_reached(const Op *op) const;
    bool poll();
    void finish(Op *op);
    Op *get_op();
    void put_ref(Op *op);
    void setup_sdma();
    std::vector<CeCopy> expand(const Op *op, size_t lanes);
};

// ------------------------------------------------------------------ set-up ---
namespace {
struct AgentSearch {
    uint32_t want_bdf;
    uint32_t want_domain;
    hsa_agent_t match, first_gpu;
    bool have_match = false;
    int ngpu = 0;
};

hsa_status_t agent_cb(hsa_agent_t a, void *data) {
    AgentSearch *s = static_cast<AgentSearch *>(data);
    hsa_device_type_t t;
    if (hsa_agent_get_info(a, HSA_AGENT_INFO_DEVICE, &t) != HSA_STATUS_SUCCESS) return HSA_STATUS_SUCCESS;
    if (t != HSA_DEVICE_TYPE_GPU) return HSA_STATUS_SUCCESS;
    if (s->ngpu++ == 0) s->first_gpu = a;
    uint32_t bdf = 0, domain = 0;
    if (hsa_agent_get_info(a, (hsa_agent_info_t)HSA_AMD_AGENT_INFO_BDFID, &bdf) == HSA_STATUS_SUCCESS &&
        hsa_agent_get_info(a, (hsa_agent_info_t)HSA_AMD_AGENT_INFO_DOMAIN, &domain) == HSA_STATUS_SUCCESS &&
        bdf == s->want_bdf && domain == s->want_domain) {
        s->match = a;
        s->have_match = true;
    }
    return HSA_STATUS_SUCCESS;
}
}  // namespace

void Proxy::setup_sdma() {
    int can = 0;
    if (hipDeviceGetAttribute(&can, hipDeviceAttributeCanUseStreamWaitValue, device) != hipSuccess || !can) {
        sdma_why = "the device does not support stream wait-value operations";
        return;
    }
    if (hsa_init() != HSA_STATUS_SUCCESS) {
        sdma_why = "hsa_init failed";
        return;
    }
    hsa_up = true;
    char bus[64] = {0};
    AgentSearch s{};
    unsigned dom = 0, b = 0, d = 0, f = 0;
    if (hipDeviceGetPCIBusId(bus, sizeof(bus), device) == hipSuccess &&
        sscanf(bus, "%x:%x:%x.%x", &dom, &b, &d, &f) == 4) {
        s.want_domain = dom;
        s.want_bdf = (b << 8) | (d << 3) | f;
    } else {
        s.want_bdf = 0xffffffffu;
    }
    hsa_iterate_agents(agent_cb, &s);
    if (s.have_match) agent = s.match;
    else if (s.ngpu == 1) agent = s.first_gpu;
    else {
        sdma_why = "could not identify the HSA agent of the device";
        return;
    }
    if (hipMalloc(&warm, 8192) != hipSuccess) {
        sdma_why = "could not allocate the engine warm-up buffer";
        return;
    }
    // Try every engine id once with a tiny copy: ids the runtime rejects are left
    // out, and the first use of an engine (queue creation, milliseconds) is paid here.
    hsa_signal_t sig;
    if (hsa_signal_create(1, 0, nullptr, &sig) != HSA_STATUS_SUCCESS) {
        sdma_why = "hsa_signal_create failed";
        return;
    }
    for (int i = 0; i < kMaxEngines; ++i) {
        hsa_signal_store_relaxed(sig, 1);
        hsa_status_t st = hsa_amd_memory_async_copy_on_engine(
            (char *)warm + 4096, agent, warm, agent, 256, 0, nullptr, sig,
            (hsa_amd_sdma_engine_id_t)(1u << i), true);
        if (st != HSA_STATUS_SUCCESS) continue;
        if (hsa_signal_wait_scacquire(sig, HSA_SIGNAL_CONDITION_LT, 1, 4000000000ull,
                                      HSA_WAIT_STATE_BLOCKED) >= 1)
            continue;   // never completed within 4 s: do not use this engine
        engine_bit[nengines++] = 1u << i;
    }
    hsa_signal_destroy(sig);
    if (nengines == 0) {
        sdma_why = "no SDMA engine accepted a copy";
        return;
    }
    sdma_ok = true;
}

// Signal words (device memory the caller's stream waits on) are never given back to
// the allocator: memory of that kind that a stream operation has read is kept until
// the process ends, and a context created later takes the words over together with
// the last sequence number each one holds.
namespace {
struct SignalWord {
    uint64_t *word;
    uint64_t seq;
    int device;
};
std::mutex g_signal_mu;
std::vector<SignalWord> g_signal_pool;
}  // namespace

Op *Proxy::get_op() {  // mu held
    if (!free_ops.empty()) {
        Op *op = free_ops.back();
        free_ops.pop_back();
        return op;
    }
    Op *op = new Op;
    bool ok = hipEventCreateWithFlags(&op->ready, hipEventDisableTiming) == hipSuccess;
    for (int i = 0; ok && i < kMaxStreams; ++i)
        ok = hipEventCreateWithFlags(&op->done[i], hipEventDisableTiming) == hipSuccess;
    if (ok && sdma_ok) {
        ok = hipHostMalloc((void **)&op->ready_word, 64, hipHostMallocDefault) == hipSuccess;
        if (ok) *op->ready_word = 0;
        if (ok) {
            std::lock_guard<std::mutex> lk(g_signal_mu);
            for (size_t i = 0; i < g_signal_pool.size(); ++i) {
                if (g_signal_pool[i].device != device) continue;
                op->done_word = g_signal_pool[i].word;
                op->seq = g_signal_pool[i].seq;   // the word holds this value: later numbers are fresh
                g_signal_pool[i] = g_signal_pool.back();
                g_signal_pool.pop_back();
                break;
            }
        }
        if (ok && !op->done_word) {
            ok = hipExtMallocWithFlags((void **)&op->done_word, 8, hipMallocSignalMemory) == hipSuccess;
            if (ok) __atomic_store_n(op->done_word, (uint64_t)0, __ATOMIC_RELEASE);
        }
        // never waited on, only loaded: a signal without a host interrupt per completed copy
        ok = ok && hsa_amd_signal_create(0, 0, nullptr, HSA_AMD_SIGNAL_AMD_GPU_ONLY, &op->left) == HSA_STATUS_SUCCESS;
    }
    if (!ok) {   // events and words of a half-built op are few and leak only on this error path
        delete op;
        return nullptr;
    }
    return op;
}

void Proxy::put_ref(Op *op) {  // mu held
    if (--op->refs == 0) {
        op->copies.clear();
        op->rects.clear();
        op->conns.clear();
        op->state = 0;
        op->sdma_failed = false;
        op->remote_role = 0;
        op->remote = nullptr;
        op->shape = 0;     // only an operation that went to the engines has one
        op->est_ns = 0;
        free_ops.push_back(op);
    }
}

// Copies are cut into pieces of at most clamp(total / (2 * lanes), 1 MiB, 16 MiB) so
// that the lanes (streams or engines) can be loaded evenly by bytes, whatever the mix
// of sizes: a skewed AlltoAllv is a few very large copies among many small ones.
std::vector<CeCopy> Proxy::expand(const Op *op, size_t lanes) {
    std::vector<CeCopy> work;
    uint64_t total = 0;
    for (const CeCopy &c : op->copies) total += c.bytes;
    uint64_t target = total / (2 * (lanes ? lanes : 1));
    if (target < kMinPiece) target = kMinPiece;
    if (target > kMaxPiece) target = kMaxPiece;
    for (const CeCopy &c : op->copies) {
        if (c.bytes == 0) continue;
        // A SendRecv copy writes to the address the receiver published in its record.
        uint8_t *dst_base = c.receiver >= 0
            ? (uint8_t *)reg[c.receiver].receiverRegAddr.load(std::memory_order_acquire)
            : (uint8_t *)c.dst;
        const uint64_t k = (c.bytes + target - 1) / target;
        const uint64_t per = ((c.bytes + k - 1) / k + 255u) & ~(uint64_t)255u;
        for (uint64_t off = 0; off < c.bytes; off += per) {
            const uint64_t n = c.bytes - off < per ? c.bytes - off : per;
            work.push_back(CeCopy{(const uint8_t *)c.src + off, dst_base + off, n, -1});
        }
    }
    return work;
}

// ------------------------------------------------------- event back end ------
void Proxy::issue_events(Op *op) {
    // Operations are issued in the order they were queued, so every earlier transfer
    // on these connections has started and the receiver proxy is free to publish.
    // (An earlier SDMA operation may still wait for its stream: keep it moving.)
    while (!receivers_ready(op)) {
        poll();
        std::this_thread::yield();
    }
    const auto t0 = std::chrono::steady_clock::now();
    int ns = op->want_streams < 1 ? 1 : (op->want_streams > max_streams ? max_streams : op->want_streams);
    std::vector<CeCopy> work = expand(op, (size_t)ns);
    if ((size_t)ns > work.size()) ns = work.empty() ? 1 : (int)work.size();
    hipError_t err = hipSuccess;
    for (int i = 0; i < ns && err == hipSuccess; ++i) err = hipStreamWaitEvent(streams[i], op->ready, 0);
    mark_started(op);
    uint64_t load[kMaxStreams] = {};
    const hipMemcpyKind kind =
        op->kind == VCCL_CE_HIP_NOCU ? hipMemcpyDeviceToDeviceNoCU : hipMemcpyDeviceToDevice;
    uint64_t bytes = 0;
    for (size_t j = 0; j < work.size() && err == hipSuccess; ++j) {
        int best = 0;
        for (int i = 1; i < ns; ++i)
            if (load[i] < load[best]) best = i;
        err = hipMemcpyAsync(work[j].dst, work[j].src, work[j].bytes, kind, streams[best]);
        load[best] += work[j].bytes;
        bytes += work[j].bytes;
    }
    for (int i = 0; i < ns && err == hipSuccess; ++i) err = hipEventRecord(op->done[i], streams[i]);
    const auto t1 = std::chrono::steady_clock::now();
    n_ops.fetch_add(1, std::memory_order_relaxed);
    n_copies.fetch_add(work.size(), std::memory_order_relaxed);
    n_bytes.fetch_add(bytes, std::memory_order_relaxed);
    issue_ns.fetch_add((uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(t1 - t0).count(),
                       std::memory_order_relaxed);
    {
        std::lock_guard<std::mutex> lk(mu);
        op->nstreams = ns;
        op->err = err;
        op->state = err == hipSuccess ? 1 : 2;
    }
    cv_issued.notify_all();
    if (err == hipSuccess) {
        op->monitor_id = ++next_monitor_id;
        (void)vccl_monitor_post(monitor[op->primitive], op->monitor_id, bytes, now_ns());
        pending.push_back(op);
    } else {
        std::lock_guard<std::mutex> lk(mu);
        --in_flight;
        put_ref(op);
        cv_idle.notify_all();
    }
}

// -------------------------------------------------------- sdma back end ------
// Returns false while the caller's stream has not yet reached the operation.
bool Proxy::stream_reached(const Op *op) const {
    if (op->ready_event) return hipEventQuery(op->ready) != hipErrorNotReady;
    return __atomic_load_n(op->ready_word, __ATOMIC_ACQUIRE) >= op->seq;
}

// Receiving side of a cross-process transfer: once the caller's stream has reached the
// operation (the buffer may be overwritten) and the previous transfer of the connection
// has started, publish where this one goes and raise ready.  The operation then stays
// pending until the sender's process marks it done.
bool Proxy::issue_remote_recv(Op *op) {
    if (!stream_reached(op)) return false;
    P2pShared *sh = op->remote;
    if (sh->copyStarted.load(std::memory_order_acquire) != op->remote_seq - 1) return false;
    sh->receiverRegOffset.store(op->remote_offset, std::memory_order_relaxed);
    sh->receiverRegBytes.store(op->remote_bytes, std::memory_order_relaxed);
    sh->receiverReady.store(op->remote_seq, std::memory_order_release);
    op->bytes = 0;
    op->t_issue_ns = now_ns();
    op->monitor_id = 0;
    pending.push_back(op);
    return true;
}

bool Proxy::issue_sdma(Op *op) {
    if (op->remote_role && op->remote->aborted.load(std::memory_order_acquire)) {
        // the connection was given up: nothing is copied, the stream is released, the failure is counted
        op->copies.clear();
        op->sdma_failed = true;
        op->remote_role = 3;                       // neither side's protocol step is taken any more
        hsa_signal_store_relaxed(op->left, 0);
        op->bytes = 0;
        op->t_issue_ns = now_ns();
        op->monitor_id = 0;
        pending.push_back(op);
        return true;
    }
    if (op->remote_role == 2) return issue_remote_recv(op);
    if (!stream_reached(op)) return false;
    if (op->remote_role == 1) {
        // sender over a cross-process connection: wait for the receiver's ready, read the
        // destination from the record, mark started
        P2pShared *sh = op->remote;
        if (sh->receiverReady.load(std::memory_order_acquire) != op->remote_seq) return false;
        const uint64_t off = sh->receiverRegOffset.load(std::memory_order_relaxed);
        const uint64_t want = sh->receiverRegBytes.load(std::memory_order_relaxed);
        if (want != op->remote_bytes || off > sh->capacity || want > sh->capacity - off) {
            // the two sides disagree (a distributed library would hang or corrupt): copy nothing, say so
            sh->mismatches.fetch_add(1, std::memory_order_relaxed);
            op->copies.clear();
            op->sdma_failed = true;
        } else {
            for (CeCopy &c : op->copies) c.dst = op->remote_buffer + off;
        }
        sh->copyStarted.store(op->remote_seq, std::memory_order_release);
    }
    // A connection carries its transfers in the order their numbers were drawn: this
    // one goes when the receiver proxy has published its buffer.
    if (!receivers_ready(op)) return false;
    const auto t0 = std::chrono::steady_clock::now();
    const int ne = op->max_engines > 0 && op->max_engines < nengines ? op->max_engines : nengines;
    std::vector<CeCopy> work = expand(op, (size_t)ne);
    mark_started(op);
    hsa_signal_store_relaxed(op->left, (hsa_signal_value_t)(work.size() + op->rects.size()));
    uint64_t bytes = 0;
    // Pitched copies first.  One that the runtime does not take is replaced by plain copies
    // of its rows, which join the pieces below.
    size_t pitched = 0;
    double pitched_ns = 0;
    for (const CeRect &rc : op->rects) {
        hsa_pitched_ptr_t src{const_cast<void *>(rc.src), (size_t)rc.src_pitch, (size_t)(rc.src_pitch * rc.rows)};
        hsa_pitched_ptr_t dst{rc.dst, (size_t)rc.dst_pitch, (size_t)(rc.dst_pitch * rc.rows)};
        const hsa_dim3_t zero{0, 0, 0};
        const hsa_dim3_t range{(uint32_t)rc.width, (uint32_t)rc.rows, 1};
        const bool taken = !(op->refuse_mask & 0x10000u) &&
                           hsa_amd_memory_async_copy_rect(&dst, &zero, &src, &zero, &range, agent, hsaDeviceToDevice, 0,
                                                          nullptr, op->left) == HSA_STATUS_SUCCESS;
        if (taken) {
            ++pitched;
            bytes += rc.width * rc.rows;
            pitched_ns += kRectCost + (double)(rc.width * rc.rows) / kRectRate;
            continue;
        }
        hsa_signal_add_relaxed(op->left, (hsa_signal_value_t)rc.rows - 1);
        for (uint64_t i = 0; i < rc.rows; ++i)
            work.push_back(CeCopy{(const uint8_t *)rc.src + i * rc.src_pitch, (uint8_t *)rc.dst + i * rc.dst_pitch,
                                  rc.width, -1});
    }
    // Each piece goes to the engine with the fewest bytes so far (ties: rotate, so that
    // equal pieces still spread round-robin and small operations do not all start on
    // engine 0).  An engine that refuses a piece is passed over: the piece is offered to
    // the other engines in turn, and if none takes it, it is copied through the HIP
    // runtime on an internal stream before the operation is allowed to complete.
    uint64_t load[kMaxEngines] = {};
    uint32_t pieces_on[kMaxEngines] = {};
    std::vector<const CeCopy *> refused;
    auto offer = [&](const CeCopy &w, int e) {
        if (op->refuse_mask & (1u << e)) return false;
        return hsa_amd_memory_async_copy_on_engine(w.dst, agent, w.src, agent, w.bytes, 0, nullptr, op->left,
                                                   (hsa_amd_sdma_engine_id_t)engine_bit[e], true) == HSA_STATUS_SUCCESS;
    };
    for (const CeCopy &w : work) {
        int best = (int)(next_engine++ % (unsigned)ne);
        for (int i = 0; i < ne; ++i)
            if (load[i] < load[best]) best = i;
        bool taken = offer(w, best);
        for (int t = 1; t < ne && !taken; ++t) {
            best = (best + 1) % ne;
            taken = offer(w, best);
        }
        if (taken) {
            load[best] += w.bytes;
            ++pieces_on[best];
            engine_bytes[best].fetch_add(w.bytes, std::memory_order_relaxed);
        } else {
            hsa_signal_subtract_relaxed(op->left, 1);   // keep the count right so that the op still completes
            refused.push_back(&w);
        }
        bytes += w.bytes;
    }
    if (!refused.empty()) {
        n_refused.fetch_add(refused.size(), std::memory_order_relaxed);
        hipError_t e = hipSuccess;
        for (const CeCopy *w : refused)
            if (e == hipSuccess) e = hipMemcpyAsync(w->dst, w->src, w->bytes, hipMemcpyDeviceToDevice, streams[0]);
        if (e == hipSuccess) e = hipStreamSynchronize(streams[0]);
        if (e != hipSuccess) op->sdma_failed = true;    // the receive buffers are incomplete: reported by the next call
    }
    op->bytes = bytes;
    op->t_issue_ns = now_ns();
    op->t_seen_busy_ns = op->t_issue_ns;
    op->shape = shape_key(bytes, work.size() + (pitched << 32), ne);
    double est;
    auto seen = history.find(op->shape);
    if (seen != history.end()) {
        est = (double)seen->second;
    } else {
        est = (double)bytes / kAllRate;
        if ((double)work.size() * kAllCopyCost > est) est = (double)work.size() * kAllCopyCost;
        for (int i = 0; i < ne; ++i) {
            const double e = (double)load[i] / kEngineRate + (double)pieces_on[i] * kCopyCost;
            if (e > est) est = e;
        }
        if (pitched_ns > est) est = pitched_ns;
    }
    op->est_ns = (uint64_t)est;
    const auto t1 = std::chrono::steady_clock::now();
    n_ops.fetch_add(1, std::memory_order_relaxed);
    n_copies.fetch_add(work.size() + pitched, std::memory_order_relaxed);
    n_pitched.fetch_add(pitched, std::memory_order_relaxed);
    n_bytes.fetch_add(bytes, std::memory_order_relaxed);
    issue_ns.fetch_add((uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(t1 - t0).count(),
                       std::memory_order_relaxed);
    op->monitor_id = ++next_monitor_id;
    (void)vccl_monitor_post(monitor[op->primitive], op->monitor_id, bytes, now_ns());
    pending.push_back(op);
    return true;
}

// copyStarted: the sender has taken the destination out of the record; the receiver
// proxy may publish the next buffer of the connection.
void Proxy::mark_started(Op *op) {
    if (op->conns.empty()) return;
    {
        std::lock_guard<std::mutex> lk(started_mu);
        for (auto &c : op->conns) reg[c.first].copyStarted.store(c.second, std::memory_order_release);
    }
    cv_started.notify_all();
}

bool Proxy::receivers_ready(const Op *op) const {
    for (auto &c : op->conns)
        if (reg[c.first].receiverReady.load(std::memory_order_acquire) != c.second) return false;
    return true;
}

// Receiver proxy: for each posted transfer, in order, wait until the previous
// transfer on the connection has started (the sender has taken its address out of
// the record), then publish the application buffer and raise ready.
void Proxy::run_receiver() {
    for (;;) {
        RecvPost post;
        {
            std::unique_lock<std::mutex> lk(recv_mu);
            cv_recv.wait(lk, [&] { return recv_stop || !recv_queue.empty(); });
            if (recv_queue.empty()) return;   // stop, and nothing left to publish
            post = recv_queue.front();
            recv_queue.pop_front();
        }
        RegInfo &ri = reg[post.rank];
        // Poll for a short while (back-to-back transfers start within microseconds of each
        // other), then sleep until the sender proxy says that a transfer has started.
        const uint64_t t0 = now_ns();
        while (ri.copyStarted.load(std::memory_order_acquire) != post.seq - 1) {
            if (now_ns() - t0 < 20000) {
                std::this_thread::yield();
                continue;
            }
            std::unique_lock<std::mutex> lk(started_mu);
            cv_started.wait(lk, [&] { return ri.copyStarted.load(std::memory_order_acquire) == post.seq - 1; });
        }
        ri.receiverRegAddr.store(post.addr, std::memory_order_relaxed);
        ri.receiverReady.store(post.seq, std::memory_order_release);
    }
}

// What an operation took goes into the history of its shape.  The proxy knows the
// completion only to within its own polling: it lies between the last poll that found
// the operation incomplete and the one that found it complete.  A narrow interval is a
// measurement and is smoothed in; a wide one (the proxy slept through the completion)
// moves the estimate to its middle only if the estimate lay outside it, so that sleeping
// on too long an estimate cannot confirm that estimate.
void Proxy::learn(const Op *op, uint64_t t_done) {
    const uint64_t lo = op->t_seen_busy_ns - op->t_issue_ns, hi = t_done - op->t_issue_ns;
    if (hi <= lo) return;
    const uint64_t mid = lo + (hi - lo) / 2;
    auto it = history.find(op->shape);
    if (it == history.end()) {
        if (history.size() >= 4096) history.clear();
        history.emplace(op->shape, mid);
    } else if (hi - lo < 8000) {
        it->second = (3 * it->second + mid) / 4;
    } else if (it->second >= hi || it->second <= lo) {
        it->second = mid;
    }
}

void Proxy::finish(Op *op) {
    const uint64_t t_done = now_ns();
    if (op->monitor_id) (void)vccl_monitor_complete(monitor[op->primitive], op->monitor_id, t_done, nullptr);
    if (op->remote_role == 1) op->remote->copyDone.store(op->remote_seq, std::memory_order_release);
    if (op->kind == VCCL_CE_SDMA && !op->sdma_failed && op->shape) learn(op, t_done);
    for (auto &c : op->conns) reg[c.first].copyDone.store(c.second, std::memory_order_release);
    if (op->kind == VCCL_CE_SDMA) {
        if (op->sdma_failed) sdma_errors.fetch_add(1, std::memory_order_relaxed);
        // Release the caller's stream: it waits for this word to reach the sequence number.
        if (!op->host_sync) __atomic_store_n(op->done_word, op->seq, __ATOMIC_RELEASE);
    }
    std::lock_guard<std::mutex> lk(mu);
    if (op->kind == VCCL_CE_SDMA && op->host_sync) {
        op->state = op->sdma_failed ? 2 : 3;   // wakes the blocked caller
        cv_issued.notify_all();
    }
    --in_flight;
    put_ref(op);
    cv_idle.notify_all();
}

// Completion polling, as the paper's proxy does; sets copyDone.  Returns whether
// anything moved (an operation was issued or found complete).
bool Proxy::poll() {
    bool progress = false;
    for (size_t k = 0; k < waiting.size();) {
        if (issue_sdma(waiting[k])) {
            waiting[k] = waiting.back();
            waiting.pop_back();
            progress = true;
        } else {
            ++k;
        }
    }
    const uint64_t now = now_ns();
    for (size_t k = 0; k < pending.size();) {
        Op *op = pending[k];
        bool complete = true;
        if (op->remote_role == 2) {
            complete = op->remote->copyDone.load(std::memory_order_acquire) >= op->remote_seq;
            if (!complete && op->remote->aborted.load(std::memory_order_acquire)) {
                op->sdma_failed = true;
                complete = true;
            }
        } else if (op->kind == VCCL_CE_SDMA) {
            complete = hsa_signal_load_scacquire(op->left) <= 0;
        } else {
            for (int i = 0; i < op->nstreams; ++i) {
                if (hipEventQuery(op->done[i]) == hipErrorNotReady) {
                    complete = false;
                    break;
                }
            }
        }
        if (!complete) {
            op->t_seen_busy_ns = now;
            ++k;
            continue;
        }
        pending[k] = pending.back();
        pending.pop_back();
        finish(op);
        progress = true;
    }
    return progress;
}

// How long the sender proxy may sleep before its next poll (0 = keep polling).  The
// paper's proxy polls without pause; here the thread polls only where that buys
// latency: for a short while after anything has moved, and around the time a
// pending operation is expected to complete.  In between it sleeps - until shortly
// before that time for operations on the engines (halving the remaining time with each
// sleep, so that a wrong estimate costs little), in short slices for operations whose
// stream is not ready yet.
uint64_t Proxy::nap_ns(uint64_t now, uint64_t last_progress) const {
    if (always_poll.load(std::memory_order_relaxed)) return 0;
    constexpr uint64_t kSpin = 30000;          // keep polling this long after the last progress
    if (now - last_progress < kSpin) return 0;
    uint64_t nap = !waiting.empty() ? (now - last_progress < 1000000 ? 10000 : 50000) : 200000;
    for (const Op *op : pending) {
        if (op->remote_role == 2) {   // the other process sets the pace: look every 10 us, then every 50
            const uint64_t slice = now - op->t_issue_ns < 2000000 ? 10000 : 50000;
            nap = nap < slice ? nap : slice;
            continue;
        }
        if (op->kind != VCCL_CE_SDMA) return 0;   // event back end: short copies on HIP streams, polled
        const uint64_t dur = op->est_ns;
        const uint64_t margin = 10000 + dur / 32;
        const uint64_t due = op->t_issue_ns + (dur > margin ? dur - margin : 0);
        if (now >= due) {
            // due: poll; if it is late by more than a third of its length the estimate was
            // wrong, then look again every 20 us
            if (now < op->t_issue_ns + dur + dur / 3 + 20000) return 0;
            nap = nap < 20000 ? nap : 20000;
        } else {
            // not due yet: sleep half of what is left (an estimate that is too long then costs
            // at most as much again as the operation took), nothing under 10 us
            const uint64_t half = (due - now) / 2;
            if (half < 5000) return 0;
            nap = nap < half ? nap : half;
        }
    }
    return nap;
}

void Proxy::run() {
    (void)hipSetDevice(device);
    prctl(PR_SET_TIMERSLACK, 1000ul);   // short sleeps mean short sleeps (the default slack is 50 us)
    uint64_t last_progress = now_ns();
    for (;;) {
        Op *op = nullptr;
        {
            std::unique_lock<std::mutex> lk(mu);
            const bool busy = !pending.empty() || !waiting.empty();
            if (!busy) {
                cv_work.wait(lk, [&] { return stop || !queue.empty(); });
                last_progress = now_ns();
            } else if (queue.empty()) {
                const uint64_t nap = nap_ns(now_ns(), last_progress);
                if (nap) {
                    cv_work.wait_for(lk, std::chrono::nanoseconds(nap), [&] { return stop || !queue.empty(); });
                } else {
                    lk.unlock();
                    std::this_thread::yield();
                    lk.lock();
                }
            }
            if (!queue.empty()) {
                op = queue.front();
                queue.pop_front();
            } else if (stop && !busy) {
                return;
            }
        }
        bool progress = op != nullptr;
        if (op) {
            if (op->kind == VCCL_CE_SDMA) waiting.push_back(op);
            else issue_events(op);
        }
        if (poll()) progress = true;
        if (progress) last_progress = now_ns();
    }
}

Proxy *proxy_create(int device, int max_streams) {
    Proxy *p = new Proxy;
    p->device = device;
    p->max_streams = max_streams < 1 ? 1 : (max_streams > kMaxStreams ? kMaxStreams : max_streams);
    for (int i = 0; i < p->max_streams; ++i) {
        // default priority on purpose
        if (hipStreamCreateWithFlags(&p->streams[i], hipStreamNonBlocking) != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipStreamDestroy(p->streams[j]);
            delete p;
            return nullptr;
        }
    }
    p->setup_sdma();
    p->monitor[0] = vccl_monitor_create(8, 10000000ull);   // window 8, 10 ms: the paper's values
    p->monitor[1] = vccl_monitor_create(8, 10000000ull);
    p->th = std::thread([p] { p->run(); });
    p->receiver_th = std::thread([p] { p->run_receiver(); });
    return p;
}

bool proxy_sdma_available(Proxy *p, const char **why) {
    if (why) *why = p->sdma_why.c_str();
    return p->sdma_ok;
}

int proxy_engine_count(Proxy *p) { return p->nengines; }

uint64_t proxy_engine_bytes(Proxy *p, int engine) {
    return engine >= 0 && engine < p->nengines ? p->engine_bytes[engine].load() : 0;
}

int proxy_drain(Proxy *p) {
    std::unique_lock<std::mutex> lk(p->mu);
    p->cv_idle.wait(lk, [&] { return p->in_flight == 0; });
    return VCCL_OK;
}

bool proxy_drain_for(Proxy *p, double seconds) {
    std::unique_lock<std::mutex> lk(p->mu);
    return p->cv_idle.wait_for(lk, std::chrono::duration<double>(seconds), [&] { return p->in_flight == 0; });
}

void proxy_destroy(Proxy *p) {
    if (!p) return;
    proxy_drain(p);
    {
        std::lock_guard<std::mutex> lk(p->mu);
        p->stop = true;
    }
    p->cv_work.notify_all();
    if (p->th.joinable()) p->th.join();
    {
        std::lock_guard<std::mutex> lk(p->recv_mu);
        p->recv_stop = true;
    }
    p->cv_recv.notify_all();
    if (p->receiver_th.joinable()) p->receiver_th.join();
    for (int i = 0; i < p->max_streams; ++i) {
        (void)hipStreamSynchronize(p->streams[i]);
        (void)hipStreamDestroy(p->streams[i]);
    }
    (void)hipDeviceSynchronize();   // no stream still waits on a word that is about to go
    for (Op *op : p->free_ops) {
        (void)hipEventDestroy(op->ready);
        for (int i = 0; i < kMaxStreams; ++i) (void)hipEventDestroy(op->done[i]);
        if (op->ready_word) (void)hipHostFree((void *)op->ready_word);
        if (op->done_word) {
            std::lock_guard<std::mutex> lk(g_signal_mu);
            g_signal_pool.push_back(SignalWord{op->done_word, op->seq, p->device});
        }
        if (op->left.handle) hsa_signal_destroy(op->left);
        delete op;
    }
    vccl_monitor_destroy(p->monitor[0]);
    vccl_monitor_destroy(p->monitor[1]);
    if (p->warm) (void)hipFree(p->warm);
    if (p->hsa_up) hsa_shut_down();
    delete p;
}

static int submit_sdma(Proxy *p, Op *op, hipStream_t stream,
                       const std::vector<std::pair<int, void *>> *receivers);
static void publish_receivers(Proxy *p, Op *op, const std::vector<std::pair<int, void *>> &receivers);

// A copy-engine call is carried out once, by a host thread, when the stream reaches it: a
// graph that recorded the call's stream operations would replay them without the copies.
static int refuse_capture(hipStream_t stream) {
    if (!stream) return VCCL_OK;   // the null stream cannot capture
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &st) == hipSuccess && st != hipStreamCaptureStatusNone)
        return fail(VCCL_ERR_UNSUPPORTED, "copy-engine calls cannot be recorded into a graph (a host thread carries "
                                          "each call out once); use VCCL_MODE_CU on a capturing stream");
    return VCCL_OK;
}

int proxy_submit(Proxy *p, std::vector<CeCopy> &&copies, const Options &opt, hipStream_t stream,
                 const std::vector<std::pair<int, void *>> *receivers, std::vector<CeRect> *rects) {
    if (int rv = refuse_capture(stream)) return rv;
    if (rects && opt.ce_kind != VCCL_CE_SDMA) return fail(VCCL_ERR_ARG, "pitched copies need the 'sdma' back end");
    if (opt.ce_kind == VCCL_CE_SDMA && !p->sdma_ok)
        return fail(VCCL_ERR_UNSUPPORTED, "copy-engine back end 'sdma' is not available: %s",
                    p->sdma_why.c_str());
    Op *op;
    {
        std::lock_guard<std::mutex> lk(p->mu);
        op = p->get_op();
        if (!op) return fail(VCCL_ERR_HIP, "could not create the resources of a copy-engine operation");
        op->host_sync = opt.ce_kind == VCCL_CE_SDMA && opt.ce_sync == VCCL_SYNC_HOST;
        op->ready_event = op->host_sync || (opt.ce_kind == VCCL_CE_SDMA && opt.ce_sync == VCCL_SYNC_EVENT);
        op->refs = (opt.ce_kind == VCCL_CE_SDMA && !op->host_sync) ? 1 : 2;
        op->state = 0;
    }
    op->copies = std::move(copies);
    if (rects) op->rects = std::move(*rects);
    op->want_streams = opt.ce_streams;
    op->kind = opt.ce_kind;
    op->max_engines = opt.ce_max_engines;
    op->refuse_mask = (uint32_t)opt.ce_test_refuse;
    op->primitive = receivers ? 0 : 1;
    if (op->kind == VCCL_CE_SDMA) return submit_sdma(p, op, stream, receivers);

    hipError_t e = hipEventRecord(op->ready, stream);
    if (e != hipSuccess) {
        std::lock_guard<std::mutex> lk(p->mu);
        op->refs = 1;
        p->put_ref(op);
        return fail(VCCL_ERR_HIP, "hipEventRecord(ready) failed: %s", hipGetErrorString(e));
    }
    int nstreams = 0;
    hipError_t err = hipSuccess;
    std::unique_lock<std::mutex> hs(p->handshake_mu, std::defer_lock);
    if (receivers) {
        hs.lock();
        publish_receivers(p, op, *receivers);
    }
    {
        std::unique_lock<std::mutex> lk(p->mu);
        p->queue.push_back(op);
        ++p->in_flight;
        p->cv_work.notify_one();
        if (hs.owns_lock()) hs.unlock();
        p->cv_issued.wait(lk, [&] { return op->state != 0; });
        nstreams = op->nstreams;
        err = op->err;
    }
    int rv = VCCL_OK;
    if (err != hipSuccess) {
        rv = fail(VCCL_ERR_HIP, "copy-engine issue failed: %s", hipGetErrorString(err));
    } else {
        for (int i = 0; i < nstreams; ++i) {
            e = hipStreamWaitEvent(stream, op->done[i], 0);
            if (e != hipSuccess && rv == VCCL_OK)
                rv = fail(VCCL_ERR_HIP, "hipStreamWaitEvent(done) failed: %s", hipGetErrorString(e));
        }
    }
    {
        std::lock_guard<std::mutex> lk(p->mu);
        p->put_ref(op);
    }
    return rv;
}

// Calling thread's part of the handshake: draw the next sequence number of every
// connection of the operation and hand the buffers to the receiver proxy.  Called
// with handshake_mu held, which stays held until the op is queued, so that the
// numbers, the receiver proxy's queue and the sender proxy's queue agree in order.
static void publish_receivers(Proxy *p, Op *op, const std::vector<std::pair<int, void *>> &receivers) {
    {
        std::lock_guard<std::mutex> lk(p->recv_mu);
        for (auto &rc : receivers) {
            const uint64_t s = ++p->reg[rc.first].drawn;
            op->conns.emplace_back(rc.first, s);
            p->recv_queue.push_back(RecvPost{rc.first, s, rc.second});
        }
    }
    p->cv_recv.notify_one();
}

// SDMA back end without stream memory operations: the calling thread itself waits
// until the copies are done, so nothing at all is enqueued on the device except
// the `ready` event.  Zero kernels, at the price of a blocking call.
static int submit_sdma_host_sync(Proxy *p, Op *op, hipStream_t stream,
                                 const std::vector<std::pair<int, void *>> *receivers) {
    hipError_t e = hipEventRecord(op->ready, stream);
    if (e != hipSuccess) {
        std::lock_guard<std::mutex> lk(p->mu);
        op->refs = 1;
        p->put_ref(op);
        return fail(VCCL_ERR_HIP, "hipEventRecord(ready) failed: %s", hipGetErrorString(e));
    }
    std::unique_lock<std::mutex> hs(p->handshake_mu, std::defer_lock);
    if (receivers) {
        hs.lock();
        publish_receivers(p, op, *receivers);
    }
    int state;
    {
        std::unique_lock<std::mutex> lk(p->mu);
        p->queue.push_back(op);
        ++p->in_flight;
        p->cv_work.notify_one();
        if (hs.owns_lock()) hs.unlock();
        p->cv_issued.wait(lk, [&] { return op->state >= 2; });
        state = op->state;
        p->put_ref(op);
    }
    if (state == 2) return fail(VCCL_ERR_HIP, "an SDMA copy could not be submitted");
    return VCCL_OK;
}

static int submit_sdma(Proxy *p, Op *op, hipStream_t stream,
                       const std::vector<std::pair<int, void *>> *receivers) {
    if (op->host_sync) return submit_sdma_host_sync(p, op, stream, receivers);
    const uint64_t seq = ++op->seq;
    // proxyReadyEvent: the stream tells the proxy when everything before this call has
    // finished - by writing the sequence number into the ready word, or (ordering
    // "event") by an event the proxy polls, which dispatches nothing.
    hipError_t e = op->ready_event ? hipEventRecord(op->ready, stream)
                                   : hipStreamWriteValue64(stream, (void *)op->ready_word, seq, 0);
    // The stream resumes when the proxy stores the sequence number into the done word
    // (proxyOpCount back at zero).  Enqueued before the proxy gets the operation, so that
    // a failure here leaves nothing behind.
    const char *what = op->ready_event ? "hipEventRecord(ready)" : "hipStreamWriteValue64(ready)";
    if (e == hipSuccess) {
        what = "hipStreamWaitValue64(done)";
        e = hipStreamWaitValue64(stream, op->done_word, seq, hipStreamWaitValueGte, ~0ull);
    }
    if (e != hipSuccess) {   // the sequence number is spent: the words only ever grow
        std::lock_guard<std::mutex> lk(p->mu);
        p->put_ref(op);
        return fail(VCCL_ERR_HIP, "%s failed: %s", what, hipGetErrorString(e));
    }
    std::unique_lock<std::mutex> hs(p->handshake_mu, std::defer_lock);
    if (receivers) {
        hs.lock();
        publish_receivers(p, op, *receivers);
    }
    {
        std::lock_guard<std::mutex> lk(p->mu);
        p->queue.push_back(op);
        ++p->in_flight;
        p->cv_work.notify_one();
    }
    // From here on the proxy owns `op`.
    return VCCL_OK;
}

int proxy_submit_remote(Proxy *p, int role, P2pShared *sh, uint8_t *mapped_buffer, uint64_t seq, const void *src,
                        uint64_t offset, uint64_t bytes, const Options &opt, hipStream_t stream) {
    if (int rv = refuse_capture(stream)) return rv;
    if (opt.ce_kind != VCCL_CE_SDMA || !p->sdma_ok)
        return fail(VCCL_ERR_UNSUPPORTED, "cross-process SendRecv needs the 'sdma' copy-engine back end%s%s",
                    p->sdma_ok ? "" : ": ", p->sdma_ok ? "" : p->sdma_why.c_str());
    Op *op;
    {
        std::lock_guard<std::mutex> lk(p->mu);
        op = p->get_op();
        if (!op) return fail(VCCL_ERR_HIP, "could not create the resources of a copy-engine operation");
        op->host_sync = opt.ce_sync == VCCL_SYNC_HOST;
        op->ready_event = op->host_sync || opt.ce_sync == VCCL_SYNC_EVENT;
        op->refs = op->host_sync ? 2 : 1;
        op->state = 0;
    }
    op->copies.clear();
    if (role == 1 && bytes) op->copies.push_back(CeCopy{src, nullptr, bytes, -1});
    op->kind = VCCL_CE_SDMA;
    op->max_engines = opt.ce_max_engines;
    op->refuse_mask = (uint32_t)opt.ce_test_refuse;
    op->primitive = 0;
    op->remote_role = role;
    op->remote = sh;
    op->remote_buffer = mapped_buffer;
    op->remote_seq = seq;
    op->remote_offset = offset;
    op->remote_bytes = bytes;
    return submit_sdma(p, op, stream, nullptr);
}

void proxy_stats(Proxy *p, uint64_t *ops, uint64_t *copies, uint64_t *bytes, uint64_t *issue_ns) {
    if (ops) *ops = p->n_ops.load();
    if (copies) *copies = p->n_copies.load();
    if (bytes) *bytes = p->n_bytes.load();
    if (issue_ns) *issue_ns = p->issue_ns.load();
}

uint64_t proxy_sdma_errors(Proxy *p) { return p->sdma_errors.load(); }
uint64_t proxy_refused_pieces(Proxy *p) { return p->n_refused.load(); }
uint64_t proxy_pitched_copies(Proxy *p) { return p->n_pitched.load(); }

// P pitched copies run one after another on one engine; P * P plain copies spread over all
// engines but are bound by the engines' copy rate.
bool proxy_pitched_pays(int P, uint64_t block_bytes) {
    const double pitched = (double)P * (Proxy::kRectCost + (double)P * (double)block_bytes / Proxy::kRectRate);
    double plain = (double)P * (double)P * Proxy::kAllCopyCost;
    const double by_rate = (double)P * (double)P * (double)block_bytes / Proxy::kAllRate;
    if (by_rate > plain) plain = by_rate;
    return pitched < plain;
}
void proxy_set_always_poll(Proxy *p, bool on) { p->always_poll.store(on, std::memory_order_relaxed); }

// Processor time the two proxy threads have used so far (what the paper's CPU
// utilisation figure, Section 4.1, charges to the SM-free design).
int proxy_cpu_time(Proxy *p, uint64_t *sender_ns, uint64_t *receiver_ns) {
    std::thread *threads[2] = {&p->th, &p->receiver_th};
    uint64_t *out[2] = {sender_ns, receiver_ns};
    for (int i = 0; i < 2; ++i) {
        if (!out[i]) continue;
        clockid_t cid;
        struct timespec ts;
        if (pthread_getcpuclockid(threads[i]->native_handle(), &cid) != 0 || clock_gettime(cid, &ts) != 0)
            return fail(VCCL_ERR_UNSUPPORTED, "the thread's processor-time clock cannot be read");
        *out[i] = (uint64_t)ts.tv_sec * 1000000000ull + (uint64_t)ts.tv_nsec;
    }
    return VCCL_OK;
}

vccl_monitor *proxy_monitor(Proxy *p, int primitive) {
    return (primitive == 0 || primitive == 1) ? p->monitor[primitive] : nullptr;
}

int proxy_reginfo(Proxy *p, int receiver, uint64_t *ready, uint64_t *started, uint64_t *done,
                  void **addr) {
    if (receiver < 0 || receiver >= VCCL_MAX_RANKS)
        return fail(VCCL_ERR_ARG, "receiver rank %d out of range", receiver);
    RegInfo &ri = p->reg[receiver];
    if (ready) *ready = ri.receiverReady.load(std::memory_order_acquire);
    if (started) *started = ri.copyStarted.load(std::memory_order_acquire);
    if (done) *done = ri.copyDone.load(std::memory_order_acquire);
    if (addr) *addr = ri.receiverRegAddr.load(std::memory_order_acquire);
    return VCCL_OK;
}

}  // namespace vccl
