// Copy-engine path: a host proxy thread issues device-to-device copies on
// internal streams so that no kernel is launched for the transfer (the paper's
// SM-free P2P: data movement by copy engines, Section 3.2 item 1; control on the
// CPU with completion polled by event query, Section 3.2 items 1-2).
//
// Stream order (Section 3.2 item 3) is kept with events only - no spin kernel and
// no host callback (the host-function variant can deadlock because callbacks of
// independent streams may be serialised):
//   caller:  record `ready` on its stream -> hand the op to the proxy
//   proxy:   every internal stream waits on `ready`, copies are issued, `done[i]`
//            is recorded behind them
//   caller:  its stream waits on every `done[i]`, then the call returns.
// The host blocks only for the microseconds the proxy needs to enqueue the batch.
//
// For SendRecv each connection also walks the receiver-owned handshake record of
// Section 3.2 (receiverRegAddr / receiverReady -> copyStarted -> copyDone).  The
// paper's 1-bit flags are kept here as monotonically increasing sequence numbers,
// which need no reset between operations.
#include <chrono>
#include <condition_variable>
#include <deque>
#include <thread>

#include "common.h"

namespace vccl {

namespace {
constexpr int kMaxStreams = 8;

struct RegInfo {  // one per receiving rank
    std::atomic<void *> receiverRegAddr{nullptr};
    std::atomic<uint64_t> receiverReady{0};
    std::atomic<uint64_t> copyStarted{0};
    std::atomic<uint64_t> copyDone{0};
};

struct Op {
    std::vector<CeCopy> copies;
    std::vector<std::pair<int, uint64_t>> conns;  // (receiver rank, sequence number)
    hipEvent_t ready = nullptr;
    hipEvent_t done[kMaxStreams] = {};
    int nstreams = 0;          // streams this op used
    int want_streams = 1;
    bool nocu = true;
    int state = 0;             // 0 queued, 1 issued, 2 failed   (guarded by Proxy::mu)
    hipError_t err = hipSuccess;
    int refs = 0;              // caller + proxy                 (guarded by Proxy::mu)
};
}  // namespace

class Proxy {
public:
    int device = 0;
    int max_streams = kMaxStreams;
    hipStream_t streams[kMaxStreams] = {};
    std::thread th;
    std::mutex mu, handshake_mu;
    std::condition_variable cv_work, cv_issued, cv_idle;
    std::deque<Op *> queue;
    std::vector<Op *> pending;   // issued, completion not yet observed (proxy thread only)
    std::vector<Op *> free_ops;
    bool stop = false;
    size_t in_flight = 0;        // queued + pending
    RegInfo reg[VCCL_MAX_RANKS];
    std::atomic<uint64_t> n_ops{0}, n_copies{0}, n_bytes{0}, issue_ns{0};

    void run();
    void issue(Op *op);
    void poll();
    Op *get_op();
    void put_ref(Op *op);
};

Op *Proxy::get_op() {  // mu held
    if (!free_ops.empty()) {
        Op *op = free_ops.back();
        free_ops.pop_back();
        return op;
    }
    Op *op = new Op;
    if (hipEventCreateWithFlags(&op->ready, hipEventDisableTiming) != hipSuccess) {
        delete op;
        return nullptr;
    }
    for (int i = 0; i < kMaxStreams; ++i) {
        if (hipEventCreateWithFlags(&op->done[i], hipEventDisableTiming) != hipSuccess) {
            delete op;
            return nullptr;
        }
    }
    return op;
}

void Proxy::put_ref(Op *op) {  // mu held
    if (--op->refs == 0) {
        op->copies.clear();
        op->conns.clear();
        op->state = 0;
        free_ops.push_back(op);
    }
}

void Proxy::issue(Op *op) {
    const auto t0 = std::chrono::steady_clock::now();
    std::vector<CeCopy> work;
    int ns = op->want_streams < 1 ? 1 : (op->want_streams > max_streams ? max_streams : op->want_streams);
    // Few large copies: cut them so that every internal stream (engine) gets a share.
    size_t pieces = 1;
    if (!op->copies.empty() && op->copies.size() < (size_t)ns)
        pieces = ((size_t)ns + op->copies.size() - 1) / op->copies.size();
    for (const CeCopy &c : op->copies) {
        if (c.bytes == 0) continue;
        // A SendRecv copy writes to the address the receiver published in its record.
        uint8_t *dst_base = c.receiver >= 0
            ? (uint8_t *)reg[c.receiver].receiverRegAddr.load(std::memory_order_acquire)
            : (uint8_t *)c.dst;
        size_t k = pieces;
        if (c.bytes < (uint64_t)(1u << 20) * k) k = 1;
        uint64_t per = ((c.bytes + k - 1) / k + 255u) & ~(uint64_t)255u;
        for (uint64_t off = 0; off < c.bytes; off += per) {
            const uint64_t n = c.bytes - off < per ? c.bytes - off : per;
            work.push_back(CeCopy{(const uint8_t *)c.src + off, dst_base + off, n, -1});
        }
    }
    if ((size_t)ns > work.size()) ns = work.empty() ? 1 : (int)work.size();
    hipError_t err = hipSuccess;
    for (int i = 0; i < ns && err == hipSuccess; ++i) err = hipStreamWaitEvent(streams[i], op->ready, 0);
    for (auto &c : op->conns) reg[c.first].copyStarted.store(c.second, std::memory_order_release);
    uint64_t load[kMaxStreams] = {};
    const hipMemcpyKind kind = op->nocu ? hipMemcpyDeviceToDeviceNoCU : hipMemcpyDeviceToDevice;
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
        pending.push_back(op);
    } else {
        std::lock_guard<std::mutex> lk(mu);
        --in_flight;
        put_ref(op);
        cv_idle.notify_all();
    }
}

// Completion polling by event query, as the paper's proxy does; sets copyDone.
void Proxy::poll() {
    for (size_t k = 0; k < pending.size();) {
        Op *op = pending[k];
        bool complete = true;
        for (int i = 0; i < op->nstreams; ++i) {
            if (hipEventQuery(op->done[i]) == hipErrorNotReady) {
                complete = false;
                break;
            }
        }
        if (!complete) {
            ++k;
            continue;
        }
        for (auto &c : op->conns) reg[c.first].copyDone.store(c.second, std::memory_order_release);
        pending[k] = pending.back();
        pending.pop_back();
        std::lock_guard<std::mutex> lk(mu);
        --in_flight;
        put_ref(op);
        cv_idle.notify_all();
    }
}

void Proxy::run() {
    (void)hipSetDevice(device);
    for (;;) {
        Op *op = nullptr;
        {
            std::unique_lock<std::mutex> lk(mu);
            if (pending.empty()) {
                cv_work.wait(lk, [&] { return stop || !queue.empty(); });
            } else if (queue.empty()) {
                cv_work.wait_for(lk, std::chrono::microseconds(20));
            }
            if (!queue.empty()) {
                op = queue.front();
                queue.pop_front();
            } else if (stop && pending.empty()) {
                return;
            }
        }
        if (op) issue(op);
        poll();
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
    p->th = std::thread([p] { p->run(); });
    return p;
}

int proxy_drain(Proxy *p) {
    std::unique_lock<std::mutex> lk(p->mu);
    p->cv_idle.wait(lk, [&] { return p->in_flight == 0; });
    return VCCL_OK;
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
    for (int i = 0; i < p->max_streams; ++i) {
        (void)hipStreamSynchronize(p->streams[i]);
        (void)hipStreamDestroy(p->streams[i]);
    }
    for (Op *op : p->free_ops) {
        (void)hipEventDestroy(op->ready);
        for (int i = 0; i < kMaxStreams; ++i) (void)hipEventDestroy(op->done[i]);
        delete op;
    }
    delete p;
}

int proxy_submit(Proxy *p, std::vector<CeCopy> &&copies, const Options &opt, hipStream_t stream,
                 const std::vector<std::pair<int, void *>> *receivers) {
    Op *op;
    {
        std::lock_guard<std::mutex> lk(p->mu);
        op = p->get_op();
        if (!op) return fail(VCCL_ERR_HIP, "could not create events for a copy-engine operation");
        op->refs = 2;
        op->state = 0;
    }
    op->copies = std::move(copies);
    op->want_streams = opt.ce_streams;
    op->nocu = opt.ce_kind_nocu != 0;
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
        // Receiver side of the handshake: once the previous transfer on the
        // connection has started, publish the application buffer and raise ready.
        // The lock is held until the op is queued so that records and queue agree.
        hs.lock();
        for (auto &rc : *receivers) {
            RegInfo &ri = p->reg[rc.first];
            while (ri.copyStarted.load(std::memory_order_acquire) !=
                   ri.receiverReady.load(std::memory_order_relaxed))
                std::this_thread::yield();
            ri.receiverRegAddr.store(rc.second, std::memory_order_relaxed);
            const uint64_t seq = ri.receiverReady.load(std::memory_order_relaxed) + 1;
            ri.receiverReady.store(seq, std::memory_order_release);
            op->conns.emplace_back(rc.first, seq);
        }
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

void proxy_stats(Proxy *p, uint64_t *ops, uint64_t *copies, uint64_t *bytes, uint64_t *issue_ns) {
    if (ops) *ops = p->n_ops.load();
    if (copies) *copies = p->n_copies.load();
    if (bytes) *bytes = p->n_bytes.load();
    if (issue_ns) *issue_ns = p->issue_ns.load();
}

int proxy_reginfo(Proxy *p, int receiver, uint64_t *ready, uint64_t *started, uint64_t *done,
                  void **addr) {
    if (receiver < 0 || receiver >= VCCL_MAX_RANKS) return fail(VCCL_ERR_ARG, "receiver rank %d out of range", receiver);
    RegInfo &ri = p->reg[receiver];
    if (ready) *ready = ri.receiverReady.load(std::memory_order_acquire);
    if (started) *started = ri.copyStarted.load(std::memory_order_acquire);
    if (done) *done = ri.copyDone.load(std::memory_order_acquire);
    if (addr) *addr = ri.receiverRegAddr.load(std::memory_order_acquire);
    return VCCL_OK;
}

}  // namespace vccl
