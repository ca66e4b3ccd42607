// The C boundary: argument validation, the host planner that turns count /
// displacement tables into segment descriptors, and dispatch to the compute-unit
// or copy-engine path.  Primitive semantics: SendRecv and AlltoAll(v) as the
// reduction-free P2P primitives of the paper (Section 1, Challenge 1; Section 2.1).
#include <fcntl.h>
#include <signal.h>
#include <sys/mman.h>
#include <sys/stat.h>
#include <time.h>
#include <unistd.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <memory>

#include "common.h"

namespace vccl {

// ------------------------------------------------------------------ errors ---
static thread_local std::string tls_error = "";

int fail(int status, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    tls_error = buf;
    return status;
}
const char *last_error_cstr() { return tls_error.c_str(); }

// --------------------------------------------------------- descriptor ring ---
int DescRing::init(size_t cap) {
    capacity = cap;
    for (int i = 0; i < kSlots; ++i) {
        VCCL_HIP(hipHostMalloc((void **)&slot[i].host, cap * sizeof(Seg), hipHostMallocDefault));
        VCCL_HIP(hipMalloc((void **)&slot[i].dev, cap * sizeof(Seg)));
        VCCL_HIP(hipEventCreateWithFlags(&slot[i].done, hipEventDisableTiming));
        slot[i].used = false;
    }
    next = 0;
    return VCCL_OK;
}

void DescRing::destroy() {
    for (int i = 0; i < kSlots; ++i) {
        if (slot[i].done) {
            (void)hipEventSynchronize(slot[i].done);
            (void)hipEventDestroy(slot[i].done);
        }
        if (slot[i].host) (void)hipHostFree(slot[i].host);
        if (slot[i].dev) (void)hipFree(slot[i].dev);
        slot[i] = DescSlot{};
    }
    capacity = 0;
}

int DescRing::acquire(DescSlot **out) {
    DescSlot *s;
    {
        std::unique_lock<std::mutex> lk(mu);
        cv.wait(lk, [&] { return !slot[next].busy; });
        s = &slot[next];
        s->busy = true;
        next = (next + 1) % kSlots;
    }
    // A slot is recycled only after the launch that last read it has finished.
    if (s->used) {
        hipError_t e = hipEventSynchronize(s->done);
        if (e != hipSuccess) {
            release(s);
            return fail(VCCL_ERR_HIP, "hipEventSynchronize(descriptor slot) failed: %s", hipGetErrorString(e));
        }
    }
    s->used = true;
    *out = s;
    return VCCL_OK;
}

void DescRing::release(DescSlot *s) {
    {
        std::lock_guard<std::mutex> lk(mu);
        s->busy = false;
    }
    cv.notify_all();
}

// ------------------------------------------------------------------ context ---
struct Context {
    int device = 0;
    int max_ranks = 0;
    int cu_count = 0;
    Options opt;
    std::mutex opt_mu;
    DescRing ring;
    FifoPool fifo;
    MoeScratch moe;
    Proxy *proxy = nullptr;
    std::atomic<uint64_t> ce_errors_reported{0};
    bool wait_on_cp = false;   // the process asked the HIP runtime to carry out stream waits in the command processor
};

static std::mutex g_mu;
static std::shared_ptr<Context> g_ctx;

static std::shared_ptr<Context> ctx_get() {
    std::lock_guard<std::mutex> lk(g_mu);
    return g_ctx;
}

static Options options_of(Context &c) {
    std::lock_guard<std::mutex> lk(c.opt_mu);
    return c.opt;
}

// ------------------------------------------------------------------ planner ---
struct Piece {
    const uint8_t *src;
    uint8_t *dst;
    uint64_t bytes;
    int receiver;
};

// O(n log n) check that no receive piece overlaps another receive piece or any
// send piece (undefined behaviour for an exchange; rejected when "check" is on).
static int check_overlap(const std::vector<Piece> &pieces) {
    struct R {
        const uint8_t *p;
        uint64_t n;
        bool is_dst;
    };
    std::vector<R> rs;
    rs.reserve(pieces.size() * 2);
    for (const Piece &pc : pieces) {
        if (!pc.bytes) continue;
        rs.push_back(R{pc.src, pc.bytes, false});
        rs.push_back(R{pc.dst, pc.bytes, true});
    }
    std::sort(rs.begin(), rs.end(), [](const R &a, const R &b) { return a.p < b.p; });
    // sweep: remember the furthest-reaching range so far of each kind
    const uint8_t *dst_end = nullptr, *src_end = nullptr;
    for (const R &r : rs) {
        if (r.is_dst) {
            if ((dst_end && r.p < dst_end) || (src_end && r.p < src_end))
                return fail(VCCL_ERR_OVERLAP, "a receive segment at %p (+%llu) overlaps another segment",
                            (const void *)r.p, (unsigned long long)r.n);
            if (!dst_end || r.p + r.n > dst_end) dst_end = r.p + r.n;
        } else {
            if (dst_end && r.p < dst_end)
                return fail(VCCL_ERR_OVERLAP, "a send segment at %p (+%llu) overlaps a receive segment",
                            (const void *)r.p, (unsigned long long)r.n);
            if (!src_end || r.p + r.n > src_end) src_end = r.p + r.n;
        }
    }
    return VCCL_OK;
}

// An engine that refused a copy of an earlier, already returned operation cannot fail that
// call any more: the first copy-engine call after it does, once.
static int report_earlier_ce_failure(Context &c) {
    const uint64_t errs = proxy_sdma_errors(c.proxy);
    if (errs > c.ce_errors_reported.exchange(errs))
        return fail(VCCL_ERR_HIP, "an earlier copy-engine operation could not submit all of its copies "
                                  "(%llu such operations so far): its receive buffers are incomplete",
                    (unsigned long long)errs);
    return VCCL_OK;
}

// Equal-block AlltoAll on the copy engines when the buffers of one side lie at a constant
// stride (one allocation cut into P rank buffers): the P blocks that a rank sends - or
// receives - are then P rows at a constant pitch on both sides, i.e. ONE pitched copy, P of
// them for the exchange in place of P * P plain ones.  Every copy costs the engines several
// microseconds whatever its size, so for small blocks and many ranks this is what bounds
// the exchange.  The runtime runs pitched copies one after another on one engine, so they
// are used only where that is still the shorter way (proxy_pitched_pays), or always under
// option ce_pitched = 2.  Fills `rects` and returns true if the call takes this form.
static bool pitched_alltoall(void *const *sendbuf, void *const *recvbuf, uint64_t c, int P, const Options &opt,
                             std::vector<CeRect> &rects) {
    if (opt.ce_kind != VCCL_CE_SDMA || opt.ce_pitched == 0 || (c & 15u) || c > 0xffffffffull) return false;
    if (opt.ce_max_engines) return false;   // the caller limits the engines; a pitched copy cannot be told which to use
    if (opt.ce_pitched == 1 && !proxy_pitched_pays(P, c)) return false;
    auto stride_of = [&](void *const *buf, uint64_t *stride) {
        const uintptr_t b0 = reinterpret_cast<uintptr_t>(buf[0]), b1 = reinterpret_cast<uintptr_t>(buf[1]);
        if (!b0 || b1 <= b0 || ((b0 | b1) & 15u)) return false;
        const uint64_t d = b1 - b0;
        if (d < (uint64_t)P * c) return false;
        for (int r = 2; r < P; ++r)
            if (reinterpret_cast<uintptr_t>(buf[r]) != b0 + (uint64_t)r * d) return false;
        *stride = d;
        return true;
    };
    for (int r = 0; r < P; ++r)
        if (!sendbuf[r] || !recvbuf[r] || ((reinterpret_cast<uintptr_t>(sendbuf[r]) | reinterpret_cast<uintptr_t>(recvbuf[r])) & 15u))
            return false;
    uint64_t d = 0;
    rects.clear();
    if (stride_of(recvbuf, &d)) {
        // rank s: block r of send[s] -> block s of recv[r] = recv[0] + r * d + s * c
        for (int s = 0; s < P; ++s)
            rects.push_back(CeRect{sendbuf[s], (uint8_t *)recvbuf[0] + (uint64_t)s * c, c, (uint64_t)P, c, d});
        return true;
    }
    if (stride_of(sendbuf, &d)) {
        // rank r: block r of send[s] = send[0] + s * d + r * c -> block s of recv[r]
        for (int r = 0; r < P; ++r)
            rects.push_back(CeRect{(const uint8_t *)sendbuf[0] + (uint64_t)r * c, recvbuf[r], c, (uint64_t)P, d, c});
        return true;
    }
    return false;
}

static int run_pieces(Context &c, std::vector<Piece> &pieces, vccl_mode mode, hipStream_t stream,
                      const std::vector<std::pair<int, void *>> *receivers) {
    const Options opt = options_of(c);
    if (opt.check) {
        int rv = check_overlap(pieces);
        if (rv) return rv;
    }
    if (mode == VCCL_MODE_CU) {
        CopyPlan plan;
        plan.segs.reserve(pieces.size());
        for (const Piece &pc : pieces)
            if (pc.bytes) plan.segs.push_back(Seg{pc.src, pc.dst, pc.bytes, 0, 0});
        // the all-aligned kernel needs the full grid
        const bool allow_fast = opt.cu_fast_path && !opt.cu_max_wg && !opt.cu_wg_per_cu;
        int rv = plan_tiles(plan, opt.cu_unroll, opt.cu_threads, allow_fast);
        if (rv) return rv;
        return launch_copy(plan, opt, c.cu_count, c.ring, stream);
    }
    if (mode == VCCL_MODE_CE) {
        std::vector<CeCopy> copies;
        copies.reserve(pieces.size());
        for (const Piece &pc : pieces)
            if (pc.bytes) copies.push_back(CeCopy{pc.src, pc.dst, pc.bytes, pc.receiver});
        if (copies.empty()) return VCCL_OK;
        int rv = report_earlier_ce_failure(c);
        if (rv) return rv;
        return proxy_submit(c.proxy, std::move(copies), opt, stream, receivers);
    }
    return fail(VCCL_ERR_ARG, "unknown mode %d", (int)mode);
}

static int check_common(const std::shared_ptr<Context> &c, int P, const void *a, const void *b) {
    if (!c) return fail(VCCL_ERR_NOT_INIT, "vccl_init has not been called");
    if (P < 1 || P > c->max_ranks)
        return fail(VCCL_ERR_ARG, "P = %d is outside 1..max_ranks (%d)", P, c->max_ranks);
    if (!a || !b) return fail(VCCL_ERR_ARG, "buffer pointer array is NULL");
    return VCCL_OK;
}

// Validation and descriptor order of an AlltoAllv description (host only).
static int alltoallv_pieces(void *const *sendbuf, const uint64_t *sendcounts, const uint64_t *sdispls,
                            void *const *recvbuf, const uint64_t *recvcounts, const uint64_t *rdispls,
                            int P, std::vector<Piece> &pieces) {
    for (int s = 0; s < P; ++s)
        for (int r = 0; r < P; ++r)
            if (sendcounts[(size_t)s * P + r] != recvcounts[(size_t)r * P + s])
                return fail(VCCL_ERR_COUNT_MISMATCH,
                            "sendcounts[%d][%d] = %llu but recvcounts[%d][%d] = %llu", s, r,
                            (unsigned long long)sendcounts[(size_t)s * P + r], r, s,
                            (unsigned long long)recvcounts[(size_t)r * P + s]);
    pieces.clear();
    pieces.reserve((size_t)P * P);
    // Destination-major with the source rotated by the destination index: at any
    // moment the segments in flight fan out over all sources and destinations
    // instead of converging on one receiver (the incast concern of Section 6).
    for (int k = 0; k < P; ++k) {
        for (int r = 0; r < P; ++r) {
            const int s = (r + k) % P;
            const uint64_t n = recvcounts[(size_t)r * P + s];
            if (!n) continue;
            if (!sendbuf[s] || !recvbuf[r])
                return fail(VCCL_ERR_ARG, "NULL buffer for a non-empty segment %d -> %d", s, r);
            pieces.push_back(Piece{(const uint8_t *)sendbuf[s] + sdispls[(size_t)s * P + r],
                                   (uint8_t *)recvbuf[r] + rdispls[(size_t)r * P + s], n, -1});
        }
    }
    return VCCL_OK;
}

static int alltoallv_impl(Context &c, void *const *sendbuf, const uint64_t *sendcounts,
                          const uint64_t *sdispls, void *const *recvbuf, const uint64_t *recvcounts,
                          const uint64_t *rdispls, int P, vccl_mode mode, hipStream_t stream) {
    if (mode != VCCL_MODE_CU && mode != VCCL_MODE_CE)
        return fail(mode == VCCL_MODE_CU_STAGED ? VCCL_ERR_UNSUPPORTED : VCCL_ERR_ARG,
                    "mode %d is not available for AlltoAll(v)", (int)mode);
    std::vector<Piece> pieces;
    int rv = alltoallv_pieces(sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, pieces);
    if (rv) return rv;
    return run_pieces(c, pieces, mode, stream, nullptr);
}

}  // namespace vccl

using namespace vccl;

// When the library is loaded: ask the HIP runtime to carry out stream wait-value
// operations in the command processor rather than with a helper kernel, unless the
// process has already said what it wants.  The runtime reads the variable when it
// starts (the process's first HIP call), so this is in time for a program that links
// the library; a process that loads it later sets the variable itself (vccl.h).
__attribute__((constructor)) static void vccl_request_wait_on_cp() { setenv("GPU_STREAMOPS_CP_WAIT", "1", 0); }

// ================================================================= C boundary ==
extern "C" {

const char *vccl_last_error(void) { return last_error_cstr(); }

int vccl_init(int device, int max_ranks) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (g_ctx) return fail(VCCL_ERR_ARG, "vccl_init called twice without vccl_finalize");
    if (max_ranks < 1 || max_ranks > VCCL_MAX_RANKS)
        return fail(VCCL_ERR_ARG, "max_ranks = %d is outside 1..%d", max_ranks, VCCL_MAX_RANKS);
    int ndev = 0;
    VCCL_HIP(hipGetDeviceCount(&ndev));
    if (device < 0 || device >= ndev) return fail(VCCL_ERR_ARG, "device %d of %d", device, ndev);
    VCCL_HIP(hipSetDevice(device));
    auto c = std::make_shared<Context>();
    c->device = device;
    c->max_ranks = max_ranks;
    VCCL_HIP(hipDeviceGetAttribute(&c->cu_count, hipDeviceAttributeMultiprocessorCount, device));
    int rv = c->ring.init((size_t)max_ranks * (size_t)max_ranks + 8192);  // + pieces of cut segments
    if (rv) {
        c->ring.destroy();
        return rv;
    }
    rv = moe_static_scratch_init(device);   // address of the static scratch on this device
    if (rv) {
        c->ring.destroy();
        return rv;
    }
    c->proxy = proxy_create(device, 8);
    if (!c->proxy) {
        c->ring.destroy();
        return fail(VCCL_ERR_HIP, "could not create the copy-engine proxy (streams)");
    }
    // Default copy-engine back end: SDMA engines through the HSA runtime when the
    // device supports stream wait-value operations, else hipMemcpyAsync(NoCU).
    c->opt.ce_kind = proxy_sdma_available(c->proxy, nullptr) ? VCCL_CE_SDMA : VCCL_CE_HIP_NOCU;
    // Which ordering dispatches nothing depends on how the HIP runtime carries out
    // hipStreamWaitValue64: with GPU_STREAMOPS_CP_WAIT=1 in the environment when the
    // runtime started, the command processor waits on the signal word itself; otherwise
    // the runtime launches a one-lane helper kernel that holds a wavefront slot for the
    // length of the transfer.  In the first case the default pairs that wait with an
    // event for readiness ("event": no kernel at all, and the call does not block);
    // in the second the default stays "memops".
    const char *cp = getenv("GPU_STREAMOPS_CP_WAIT");
    c->wait_on_cp = cp && atoi(cp) != 0;
    if (c->opt.ce_kind == VCCL_CE_SDMA && c->wait_on_cp) c->opt.ce_sync = VCCL_SYNC_EVENT;
    g_ctx = c;
    return VCCL_OK;
}

int vccl_finalize(void) {
    std::shared_ptr<Context> c;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        c.swap(g_ctx);
    }
    if (!c) return fail(VCCL_ERR_NOT_INIT, "vccl_finalize without vccl_init");
    (void)hipSetDevice(c->device);
    (void)proxy_drain(c->proxy);
    const uint64_t errs = proxy_sdma_errors(c->proxy);
    const bool unreported = errs > c->ce_errors_reported.load();
    proxy_destroy(c->proxy);
    c->proxy = nullptr;
    (void)hipDeviceSynchronize();
    c->ring.destroy();
    c->fifo.destroy();
    c->moe.destroy();
    if (unreported)
        return fail(VCCL_ERR_HIP, "%llu copy-engine operations could not submit all of their copies",
                    (unsigned long long)errs);
    return VCCL_OK;
}

int vccl_device_cu_count(void) {
    auto c = ctx_get();
    if (!c) return fail(VCCL_ERR_NOT_INIT, "vccl_init has not been called");
    return c->cu_count;
}

static bool parse_u64(const char *v, uint64_t *out) {
    if (!v || !*v) return false;
    char *end = nullptr;
    unsigned long long x = strtoull(v, &end, 10);
    if (*end != '\0' || v[0] == '-') return false;
    *out = x;
    return true;
}

int vccl_set_option(const char *key, const char *value) {
    auto c = ctx_get();
    if (!c) return fail(VCCL_ERR_NOT_INIT, "vccl_init has not been called");
    if (!key || !value) return fail(VCCL_ERR_ARG, "NULL option key or value");
    std::lock_guard<std::mutex> lk(c->opt_mu);
    Options &o = c->opt;
    const std::string k(key);
    if (k == "ce_kind") {
        if (!strcmp(value, "sdma")) {
            const char *why = "";
            if (!proxy_sdma_available(c->proxy, &why))
                return fail(VCCL_ERR_UNSUPPORTED, "ce_kind 'sdma' is not available: %s", why);
            o.ce_kind = VCCL_CE_SDMA;
        } else if (!strcmp(value, "hip_nocu")) o.ce_kind = VCCL_CE_HIP_NOCU;
        else if (!strcmp(value, "hip_default")) o.ce_kind = VCCL_CE_HIP_DEFAULT;
        else return fail(VCCL_ERR_ARG, "ce_kind must be 'sdma', 'hip_nocu' or 'hip_default', got '%s'", value);
        return VCCL_OK;
    }
    if (k == "ce_engines" || k == "ce_errors" || k == "ce_engine_bytes" || k == "ce_wait_on_cp" || k == "ce_refused" ||
        k == "ce_pitched_copies")
        return fail(VCCL_ERR_ARG, "%s is read-only", key);
    if (k == "ce_sync") {
        if (!strcmp(value, "memops")) o.ce_sync = VCCL_SYNC_MEMOPS;
        else if (!strcmp(value, "host")) o.ce_sync = VCCL_SYNC_HOST;
        else if (!strcmp(value, "event")) o.ce_sync = VCCL_SYNC_EVENT;
        else return fail(VCCL_ERR_ARG, "ce_sync must be 'memops', 'event' or 'host', got '%s'", value);
        return VCCL_OK;
    }
    uint64_t x = 0;
    if (!parse_u64(value, &x)) return fail(VCCL_ERR_ARG, "option %s: '%s' is not a number", key, value);
    auto in = [&](uint64_t lo, uint64_t hi) { return x >= lo && x <= hi; };
    if (k == "cu_unroll") {
        if (!(x == 1 || x == 2 || x == 4 || x == 8 || x == 16))
            return fail(VCCL_ERR_ARG, "cu_unroll must be 1, 2, 4, 8 or 16");
        o.cu_unroll = (int)x;
    } else if (k == "cu_wg_per_cu") {
        if (!in(0, 16)) return fail(VCCL_ERR_ARG, "cu_wg_per_cu must be 0..16");
        o.cu_wg_per_cu = (int)x;
    } else if (k == "cu_max_wg") {
        if (!in(0, 1u << 20)) return fail(VCCL_ERR_ARG, "cu_max_wg must be 0..1048576");
        o.cu_max_wg = (int)x;
    } else if (k == "cu_nontemporal") {
        if (!in(0, 2)) return fail(VCCL_ERR_ARG, "cu_nontemporal must be 0, 1 or 2");
        o.cu_nontemporal = (int)x;
    } else if (k == "cu_threads") {
        if (!(x == 64 || x == 128 || x == 256)) return fail(VCCL_ERR_ARG, "cu_threads must be 64, 128 or 256");
        o.cu_threads = (int)x;
    } else if (k == "cu_fast_path") {
        if (!in(0, 1)) return fail(VCCL_ERR_ARG, "cu_fast_path must be 0 or 1");
        o.cu_fast_path = (int)x;
    } else if (k == "ce_streams") {
        if (!in(1, 8)) return fail(VCCL_ERR_ARG, "ce_streams must be 1..8");
        o.ce_streams = (int)x;
    } else if (k == "moe_gather_variant") {
        if (!(x == 4 || x == 8 || x == 16 || x == 108 || x == 116 || x == 208 || x == 308 || x == 408 || x == 508))
            return fail(VCCL_ERR_ARG, "moe_gather_variant must be 4, 8, 16, 108, 116, 208, 308, 408 or 508");
        o.moe_gather_variant = (int)x;
    } else if (k == "p2p_close_wait_ms") {
        if (!in(0, 3600000)) return fail(VCCL_ERR_ARG, "p2p_close_wait_ms must be 0..3600000");
        o.p2p_close_wait_ms = (int)x;
    } else if (k == "moe_unpack_variant") {
        if (!in(0, 3)) return fail(VCCL_ERR_ARG, "moe_unpack_variant must be 0..3");
        o.moe_unpack_variant = (int)x;
    } else if (k == "moe_gather_full") {
        if (!in(0, 1)) return fail(VCCL_ERR_ARG, "moe_gather_full must be 0 or 1");
        o.moe_gather_full = (int)x;
    } else if (k == "ce_max_engines") {
        if (!in(0, 16)) return fail(VCCL_ERR_ARG, "ce_max_engines must be 0..16");
        o.ce_max_engines = (int)x;
    } else if (k == "ce_proxy_poll") {
        if (!in(0, 1)) return fail(VCCL_ERR_ARG, "ce_proxy_poll must be 0 or 1");
        o.ce_proxy_poll = (int)x;
        proxy_set_always_poll(c->proxy, x != 0);
    } else if (k == "ce_pitched") {
        if (!in(0, 2)) return fail(VCCL_ERR_ARG, "ce_pitched must be 0, 1 or 2");
        o.ce_pitched = (int)x;
    } else if (k == "ce_test_refuse") {
        if (!in(0, 0x1ffff)) return fail(VCCL_ERR_ARG, "ce_test_refuse must be 0..131071");
        o.ce_test_refuse = (int)x;
    } else if (k == "check") {
        if (!in(0, 1)) return fail(VCCL_ERR_ARG, "check must be 0 or 1");
        o.check = (int)x;
    } else if (k == "fifo_chunk_bytes") {
        if (!in(4096, 64u << 20) || (x & 4095))
            return fail(VCCL_ERR_ARG, "fifo_chunk_bytes must be a multiple of 4096 in 4 KiB..64 MiB");
        o.fifo_chunk_bytes = x;
    } else if (k == "fifo_slots") {
        if (!in(1, 64)) return fail(VCCL_ERR_ARG, "fifo_slots must be 1..64");
        o.fifo_slots = (int)x;
    } else if (k == "fifo_wg_per_conn") {
        if (!in(1, 64)) return fail(VCCL_ERR_ARG, "fifo_wg_per_conn must be 1..64");
        o.fifo_wg_per_conn = (int)x;
    } else if (k == "fifo_scoped") {
        if (!in(0, 1)) return fail(VCCL_ERR_ARG, "fifo_scoped must be 0 or 1");
        o.fifo_scoped = (int)x;
    } else if (k == "fifo_spin_limit") {
        if (!in(1, 1ull << 40)) return fail(VCCL_ERR_ARG, "fifo_spin_limit must be 1..2^40");
        o.fifo_spin_limit = x;
    } else {
        return fail(VCCL_ERR_ARG, "unknown option '%s'", key);
    }
    return VCCL_OK;
}

int vccl_get_option(const char *key, char *out, int cap) {
    auto c = ctx_get();
    if (!c) return fail(VCCL_ERR_NOT_INIT, "vccl_init has not been called");
    if (!key || !out || cap < 2) return fail(VCCL_ERR_ARG, "bad arguments to vccl_get_option");
    const Options o = options_of(*c);
    const std::string k(key);
    unsigned long long v;
    if (k == "ce_kind") {
        snprintf(out, (size_t)cap, "%s", o.ce_kind == VCCL_CE_SDMA ? "sdma"
                                         : o.ce_kind == VCCL_CE_HIP_NOCU ? "hip_nocu" : "hip_default");
        return VCCL_OK;
    } else if (k == "ce_sync") {
        snprintf(out, (size_t)cap, "%s", o.ce_sync == VCCL_SYNC_HOST ? "host"
                                         : o.ce_sync == VCCL_SYNC_EVENT ? "event" : "memops");
        return VCCL_OK;
    } else if (k == "ce_engine_bytes") {
        std::string txt;
        for (int i = 0; i < proxy_engine_count(c->proxy); ++i)
            txt += (i ? "," : "") + std::to_string((unsigned long long)proxy_engine_bytes(c->proxy, i));
        if ((int)txt.size() + 1 > cap) return fail(VCCL_ERR_ARG, "ce_engine_bytes needs %zu characters", txt.size() + 1);
        snprintf(out, (size_t)cap, "%s", txt.c_str());
        return VCCL_OK;
    } else if (k == "ce_engines") v = (unsigned long long)proxy_engine_count(c->proxy);
    else if (k == "ce_errors") v = (unsigned long long)proxy_sdma_errors(c->proxy);
    else if (k == "ce_wait_on_cp") v = c->wait_on_cp ? 1 : 0;
    else if (k == "ce_refused") v = (unsigned long long)proxy_refused_pieces(c->proxy);
    else if (k == "ce_test_refuse") v = o.ce_test_refuse;
    else if (k == "ce_pitched") v = o.ce_pitched;
    else if (k == "ce_pitched_copies") v = (unsigned long long)proxy_pitched_copies(c->proxy);
    else if (k == "ce_proxy_poll") v = o.ce_proxy_poll;
    else if (k == "cu_unroll") v = o.cu_unroll;
    else if (k == "cu_wg_per_cu") v = o.cu_wg_per_cu;
    else if (k == "cu_max_wg") v = o.cu_max_wg;
    else if (k == "cu_nontemporal") v = o.cu_nontemporal;
    else if (k == "cu_threads") v = o.cu_threads;
    else if (k == "cu_fast_path") v = o.cu_fast_path;
    else if (k == "ce_streams") v = o.ce_streams;
    else if (k == "moe_gather_variant") v = o.moe_gather_variant;
    else if (k == "moe_unpack_variant") v = o.moe_unpack_variant;
    else if (k == "p2p_close_wait_ms") v = o.p2p_close_wait_ms;
    else if (k == "moe_gather_full") v = o.moe_gather_full;
    else if (k == "ce_max_engines") v = o.ce_max_engines;
    else if (k == "check") v = o.check;
    else if (k == "fifo_chunk_bytes") v = o.fifo_chunk_bytes;
    else if (k == "fifo_slots") v = o.fifo_slots;
    else if (k == "fifo_wg_per_conn") v = o.fifo_wg_per_conn;
    else if (k == "fifo_spin_limit") v = o.fifo_spin_limit;
    else if (k == "fifo_scoped") v = o.fifo_scoped;
    else return fail(VCCL_ERR_ARG, "unknown option '%s'", key);
    snprintf(out, (size_t)cap, "%llu", v);
    return VCCL_OK;
}

int vccl_alltoallv(void *const *sendbuf, const uint64_t *sendcounts, const uint64_t *sdispls,
                   void *const *recvbuf, const uint64_t *recvcounts, const uint64_t *rdispls, int P,
                   vccl_mode mode, void *stream) {
    auto c = ctx_get();
    int rv = check_common(c, P, sendbuf, recvbuf);
    if (rv) return rv;
    if (!sendcounts || !sdispls || !recvcounts || !rdispls)
        return fail(VCCL_ERR_ARG, "count or displacement table is NULL");
    return alltoallv_impl(*c, sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, mode,
                          (hipStream_t)stream);
}

int vccl_alltoall(void *const *sendbuf, void *const *recvbuf, uint64_t bytes_per_peer, int P,
                  vccl_mode mode, void *stream) {
    auto c = ctx_get();
    int rv = check_common(c, P, sendbuf, recvbuf);
    if (rv) return rv;
    if (mode == VCCL_MODE_CU && P > 8) {   // up to 64 descriptors already ride in the kernel arguments
        const Options opt = options_of(*c);
        if (uniform_alltoall_applies(sendbuf, recvbuf, bytes_per_peer, P, opt))
            return launch_uniform_alltoall(sendbuf, recvbuf, bytes_per_peer, P, opt, (hipStream_t)stream);
    }
    if (mode == VCCL_MODE_CE && P >= 2 && bytes_per_peer) {
        std::vector<CeRect> rects;
        const Options opt = options_of(*c);
        if (pitched_alltoall(sendbuf, recvbuf, bytes_per_peer, P, opt, rects)) {
            if (opt.check) {   // the same validation as on the general path
                std::vector<Piece> pieces;
                for (int a = 0; a < P; ++a)
                    for (int b = 0; b < P; ++b)
                        pieces.push_back(Piece{(const uint8_t *)sendbuf[a] + (uint64_t)b * bytes_per_peer,
                                               (uint8_t *)recvbuf[b] + (uint64_t)a * bytes_per_peer, bytes_per_peer, -1});
                rv = check_overlap(pieces);
                if (rv) return rv;
            }
            rv = report_earlier_ce_failure(*c);
            if (rv) return rv;
            return proxy_submit(c->proxy, std::vector<CeCopy>(), opt, (hipStream_t)stream, nullptr, &rects);
        }
    }
    std::vector<uint64_t> cnt((size_t)P * P, bytes_per_peer), dsp((size_t)P * P);
    for (int a = 0; a < P; ++a)
        for (int b = 0; b < P; ++b) dsp[(size_t)a * P + b] = (uint64_t)b * bytes_per_peer;
    return alltoallv_impl(*c, sendbuf, cnt.data(), dsp.data(), recvbuf, cnt.data(), dsp.data(), P,
                          mode, (hipStream_t)stream);
}

int vccl_sendrecv(void *const *sendbuf, const uint64_t *sendbytes, const int *send_to,
                  void *const *recvbuf, const uint64_t *recvbytes, const int *recv_from, int P,
                  vccl_mode mode, void *stream) {
    auto c = ctx_get();
    int rv = check_common(c, P, sendbuf, recvbuf);
    if (rv) return rv;
    if (!sendbytes || !send_to || !recvbytes || !recv_from)
        return fail(VCCL_ERR_ARG, "size or peer table is NULL");
    if (mode != VCCL_MODE_CU && mode != VCCL_MODE_CE && mode != VCCL_MODE_CU_STAGED)
        return fail(VCCL_ERR_ARG, "unknown mode %d", (int)mode);
    for (int s = 0; s < P; ++s) {
        const int r = send_to[s];
        if (r < 0 || r >= P) return fail(VCCL_ERR_ARG, "send_to[%d] = %d is not a rank", s, r);
        if (recv_from[r] != s)
            return fail(VCCL_ERR_ARG, "recv_from[%d] = %d does not invert send_to[%d] = %d", r,
                        recv_from[r], s, r);
        if (sendbytes[s] != recvbytes[r])
            return fail(VCCL_ERR_COUNT_MISMATCH, "rank %d sends %llu bytes but rank %d expects %llu",
                        s, (unsigned long long)sendbytes[s], r, (unsigned long long)recvbytes[r]);
        if (sendbytes[s] && (!sendbuf[s] || !recvbuf[r]))
            return fail(VCCL_ERR_ARG, "NULL buffer on connection %d -> %d", s, r);
    }
    if (mode == VCCL_MODE_CU_STAGED) {
        const Options opt = options_of(*c);
        std::vector<FifoConn> conns;
        std::vector<Piece> pieces;
        for (int s = 0; s < P; ++s) {
            if (!sendbytes[s]) continue;
            conns.push_back(FifoConn{(const uint8_t *)sendbuf[s], (uint8_t *)recvbuf[send_to[s]],
                                     sendbytes[s]});
            pieces.push_back(Piece{conns.back().src, conns.back().dst, sendbytes[s], -1});
        }
        if (opt.check) {
            rv = check_overlap(pieces);
            if (rv) return rv;
        }
        if (conns.empty()) return VCCL_OK;
        return launch_fifo(c->fifo, conns, opt, c->cu_count, (hipStream_t)stream);
    }
    std::vector<Piece> pieces;
    std::vector<std::pair<int, void *>> receivers;
    for (int s = 0; s < P; ++s) {
        if (!sendbytes[s]) continue;
        const int r = send_to[s];
        pieces.push_back(Piece{(const uint8_t *)sendbuf[s], (uint8_t *)recvbuf[r], sendbytes[s],
                               mode == VCCL_MODE_CE ? r : -1});
        if (mode == VCCL_MODE_CE) receivers.emplace_back(r, recvbuf[r]);
    }
    return run_pieces(*c, pieces, mode, (hipStream_t)stream,
                      mode == VCCL_MODE_CE ? &receivers : nullptr);
}

static int moe_pack_common(const void *const *x, const int32_t *const *expert_ids, int P, int tokens, int topk,
                           uint64_t row_bytes, int num_experts, int experts_per_rank, void *const *packed,
                           uint64_t *counts_dev, uint64_t *counts_host, uint32_t *const *slot_row,
                           uint32_t *bad_ids_dev, void *stream) {
    auto c = ctx_get();
    int rv = check_common(c, P, x, packed);
    if (rv) return rv;
    if (!expert_ids || !counts_dev) return fail(VCCL_ERR_ARG, "expert_ids or counts_dev is NULL");
    if (tokens < 0 || topk < 1 || topk > 64)
        return fail(VCCL_ERR_ARG, "tokens = %d, topk = %d (topk must be 1..64)", tokens, topk);
    if (num_experts < 1 || num_experts > 1024)
        return fail(VCCL_ERR_ARG, "num_experts = %d is outside 1..1024", num_experts);
    if (row_bytes == 0 || (row_bytes & 15u))
        return fail(VCCL_ERR_ARG, "row_bytes = %llu must be a positive multiple of 16",
                    (unsigned long long)row_bytes);
    if ((uint64_t)tokens * (uint64_t)topk > 0x7fffffffull)
        return fail(VCCL_ERR_UNSUPPORTED, "more than 2^31 (token, slot) pairs per rank");
    for (int s = 0; s < P; ++s) {
        if (tokens && (!x[s] || !expert_ids[s] || !packed[s]))
            return fail(VCCL_ERR_ARG, "NULL buffer for rank %d", s);
        if ((reinterpret_cast<uintptr_t>(x[s]) | reinterpret_cast<uintptr_t>(packed[s])) & 15u)
            return fail(VCCL_ERR_ARG, "x / packed of rank %d are not 16-byte aligned", s);
    }
    return launch_moe_pack(c->moe, x, expert_ids, P, tokens, topk, row_bytes, num_experts, experts_per_rank,
                           packed, counts_dev, counts_host, slot_row, bad_ids_dev,
                           options_of(*c).moe_gather_variant, options_of(*c).moe_gather_full,
                           (hipStream_t)stream);
}

int vccl_moe_pack(const void *const *x, const int32_t *const *expert_ids, int P, int tokens, int topk,
                  uint64_t row_bytes, int num_experts, void *const *packed, uint64_t *counts_dev,
                  uint64_t *counts_host, uint32_t *bad_ids_dev, void *stream) {
    return moe_pack_common(x, expert_ids, P, tokens, topk, row_bytes, num_experts, 0, packed, counts_dev,
                           counts_host, nullptr, bad_ids_dev, stream);
}

int vccl_moe_pack_noalloc(const void *const *x, const int32_t *const *expert_ids, int P, int tokens, int topk,
                          uint64_t row_bytes, int num_experts, void *const *packed, uint64_t *counts_dev,
                          uint32_t *bad_ids_dev, void *stream) {
    auto c = ctx_get();
    int rv = check_common(c, P, x, packed);
    if (rv) return rv;
    if (!expert_ids || !counts_dev) return fail(VCCL_ERR_ARG, "expert_ids or counts_dev is NULL");
    if (tokens < 0 || topk < 1 || topk > 64)
        return fail(VCCL_ERR_ARG, "tokens = %d, topk = %d (topk must be 1..64)", tokens, topk);
    if (num_experts < 1 || num_experts > 1024)
        return fail(VCCL_ERR_ARG, "num_experts = %d is outside 1..1024", num_experts);
    if (row_bytes == 0 || (row_bytes & 15u))
        return fail(VCCL_ERR_ARG, "row_bytes = %llu must be a positive multiple of 16",
                    (unsigned long long)row_bytes);
    if ((uint64_t)tokens * (uint64_t)topk > 0x7fffffffull)
        return fail(VCCL_ERR_UNSUPPORTED, "more than 2^31 (token, slot) pairs per rank");
    for (int s = 0; s < P; ++s) {
        if (tokens && (!x[s] || !expert_ids[s] || !packed[s]))
            return fail(VCCL_ERR_ARG, "NULL buffer for rank %d", s);
        if ((reinterpret_cast<uintptr_t>(x[s]) | reinterpret_cast<uintptr_t>(packed[s])) & 15u)
            return fail(VCCL_ERR_ARG, "x / packed of rank %d are not 16-byte aligned", s);
    }
    return launch_moe_pack_noalloc(c->device, x, expert_ids, P, tokens, topk, row_bytes, num_experts, packed,
                                   counts_dev, bad_ids_dev, options_of(*c).moe_gather_variant,
                                   options_of(*c).moe_gather_full, (hipStream_t)stream);
}

int vccl_moe_pack_per_rank(const void *const *x, const int32_t *const *expert_ids, int P, int tokens, int topk,
                           uint64_t row_bytes, int num_experts, int experts_per_rank, void *const *packed,
                           uint64_t *counts_dev, uint64_t *counts_host, uint32_t *const *slot_row,
                           uint32_t *bad_ids_dev, void *stream) {
    if (experts_per_rank < 1 || num_experts < 1 || num_experts % experts_per_rank)
        return fail(VCCL_ERR_ARG, "experts_per_rank = %d does not divide num_experts = %d", experts_per_rank,
                    num_experts);
    return moe_pack_common(x, expert_ids, P, tokens, topk, row_bytes, num_experts, experts_per_rank, packed,
                           counts_dev, counts_host, slot_row, bad_ids_dev, stream);
}

int vccl_moe_dispatch_fused(const void *const *x, const int32_t *const *expert_ids, int P, int tokens, int topk,
                            uint64_t row_bytes, int num_experts, int experts_per_rank, void *const *recv,
                            const uint64_t *recv_capacity_rows, uint64_t *counts_dev, uint64_t *layout_dev,
                            uint64_t *layout_host, uint32_t *status_dev, void *stream) {
    auto c = ctx_get();
    int rv = check_common(c, P, x, recv);
    if (rv) return rv;
    if (!expert_ids || !recv_capacity_rows || !layout_dev)
        return fail(VCCL_ERR_ARG, "expert_ids, recv_capacity_rows or layout_dev is NULL");
    if (tokens < 0 || topk < 1 || topk > 64)
        return fail(VCCL_ERR_ARG, "tokens = %d, topk = %d (topk must be 1..64)", tokens, topk);
    if (num_experts < 1 || num_experts > 1024 || experts_per_rank < 1 || num_experts != P * experts_per_rank)
        return fail(VCCL_ERR_ARG, "num_experts = %d must be P * experts_per_rank = %d * %d (at most 1024)",
                    num_experts, P, experts_per_rank);
    if (row_bytes == 0 || (row_bytes & 15u))
        return fail(VCCL_ERR_ARG, "row_bytes = %llu must be a positive multiple of 16",
                    (unsigned long long)row_bytes);
    if ((uint64_t)tokens * (uint64_t)topk > 0x7fffffffull)
        return fail(VCCL_ERR_UNSUPPORTED, "more than 2^31 (token, slot) pairs per rank");
    for (int s = 0; s < P; ++s) {
        if (tokens && (!x[s] || !expert_ids[s]))
            return fail(VCCL_ERR_ARG, "NULL buffer for rank %d", s);
        if (recv_capacity_rows[s] && !recv[s])
            return fail(VCCL_ERR_ARG, "NULL receive buffer with a capacity of %llu rows for rank %d",
                        (unsigned long long)recv_capacity_rows[s], s);
        if ((reinterpret_cast<uintptr_t>(x[s]) | reinterpret_cast<uintptr_t>(recv[s])) & 15u)
            return fail(VCCL_ERR_ARG, "x / recv of rank %d are not 16-byte aligned", s);
    }
    return launch_moe_dispatch_fused(c->moe, x, expert_ids, P, tokens, topk, row_bytes, num_experts,
                                     experts_per_rank, recv, recv_capacity_rows, counts_dev, layout_dev,
                                     layout_host, status_dev, options_of(*c).moe_gather_full,
                                     (hipStream_t)stream);
}

int vccl_moe_combine_fused(const void *const *back, const uint64_t *back_capacity_rows,
                           const int32_t *const *expert_ids, int P, int tokens, int topk, uint64_t row_bytes,
                           int num_experts, int experts_per_rank, void *const *out, void *stream) {
    auto c = ctx_get();
    int rv = check_common(c, P, back, out);
    if (rv) return rv;
    if (!expert_ids || !back_capacity_rows) return fail(VCCL_ERR_ARG, "expert_ids or back_capacity_rows is NULL");
    if (tokens < 0 || topk < 1 || topk > 64)
        return fail(VCCL_ERR_ARG, "tokens = %d, topk = %d (topk must be 1..64)", tokens, topk);
    if (num_experts < 1 || num_experts > 1024 || experts_per_rank < 1 || num_experts != P * experts_per_rank)
        return fail(VCCL_ERR_ARG, "num_experts = %d must be P * experts_per_rank = %d * %d (at most 1024)",
                    num_experts, P, experts_per_rank);
    if (row_bytes == 0 || (row_bytes & 15u))
        return fail(VCCL_ERR_ARG, "row_bytes = %llu must be a positive multiple of 16",
                    (unsigned long long)row_bytes);
    if ((uint64_t)tokens * (uint64_t)topk > 0x7fffffffull)
        return fail(VCCL_ERR_UNSUPPORTED, "more than 2^31 (token, slot) pairs per rank");
    for (int s = 0; s < P; ++s) {
        if (tokens && (!expert_ids[s] || !out[s])) return fail(VCCL_ERR_ARG, "NULL buffer for rank %d", s);
        if (back_capacity_rows[s] && !back[s])
            return fail(VCCL_ERR_ARG, "NULL buffer with a capacity of %llu rows for rank %d",
                        (unsigned long long)back_capacity_rows[s], s);
        if ((reinterpret_cast<uintptr_t>(back[s]) | reinterpret_cast<uintptr_t>(out[s])) & 15u)
            return fail(VCCL_ERR_ARG, "back / out of rank %d are not 16-byte aligned", s);
    }
    return launch_moe_combine_fused(c->moe, back, back_capacity_rows, expert_ids, P, tokens, topk, row_bytes,
                                    num_experts, experts_per_rank, out, (hipStream_t)stream);
}

int vccl_moe_unpack(const void *const *packed, const int32_t *const *expert_ids, int P, int tokens,
                    int topk, uint64_t row_bytes, int num_experts, void *const *out, void *stream) {
    auto c = ctx_get();
    int rv = check_common(c, P, packed, out);
    if (rv) return rv;
    if (!expert_ids) return fail(VCCL_ERR_ARG, "expert_ids is NULL");
    if (tokens < 0 || topk < 1 || topk > 64)
        return fail(VCCL_ERR_ARG, "tokens = %d, topk = %d (topk must be 1..64)", tokens, topk);
    if (num_experts < 1 || num_experts > 1024)
        return fail(VCCL_ERR_ARG, "num_experts = %d is outside 1..1024", num_experts);
    if (row_bytes == 0 || (row_bytes & 15u))
        return fail(VCCL_ERR_ARG, "row_bytes = %llu must be a positive multiple of 16",
                    (unsigned long long)row_bytes);
    if ((uint64_t)tokens * (uint64_t)topk > 0x7fffffffull)
        return fail(VCCL_ERR_UNSUPPORTED, "more than 2^31 (token, slot) pairs per rank");
    for (int s = 0; s < P; ++s) {
        if (tokens && (!packed[s] || !expert_ids[s] || !out[s]))
            return fail(VCCL_ERR_ARG, "NULL buffer for rank %d", s);
        if ((reinterpret_cast<uintptr_t>(packed[s]) | reinterpret_cast<uintptr_t>(out[s])) & 15u)
            return fail(VCCL_ERR_ARG, "packed / out of rank %d are not 16-byte aligned", s);
    }
    return launch_moe_unpack(c->moe, packed, expert_ids, P, tokens, topk, row_bytes, num_experts, out,
                             options_of(*c).moe_unpack_variant, (hipStream_t)stream);
}

int vccl_moe_exchange_layout(const uint64_t *counts, int P, int num_experts, int experts_per_rank,
                             uint64_t row_bytes, uint64_t *sendcounts, uint64_t *sdispls,
                             uint64_t *recvcounts, uint64_t *rdispls) {
    if (!counts || !sendcounts || !sdispls || !recvcounts || !rdispls)
        return fail(VCCL_ERR_ARG, "NULL table");
    if (P < 1 || experts_per_rank < 1 || (int64_t)P * experts_per_rank != num_experts)
        return fail(VCCL_ERR_ARG, "num_experts (%d) must equal P (%d) x experts_per_rank (%d)",
                    num_experts, P, experts_per_rank);
    // Rows of one source rank are already grouped by destination, so the send
    // displacements are a running sum along the row of the rank-to-rank matrix.
    std::vector<uint64_t> rows((size_t)P * P, 0);
    for (int s = 0; s < P; ++s) {
        const uint64_t *cs = counts + (size_t)s * num_experts;
        uint64_t run = 0;
        for (int r = 0; r < P; ++r) {
            uint64_t n = 0;
            for (int j = 0; j < experts_per_rank; ++j) n += cs[(size_t)r * experts_per_rank + j];
            rows[(size_t)s * P + r] = n;
            sendcounts[(size_t)s * P + r] = n * row_bytes;
            sdispls[(size_t)s * P + r] = run;
            run += n * row_bytes;
        }
    }
    // A receiver lays incoming segments out in source-rank order.
    for (int r = 0; r < P; ++r) {
        uint64_t run = 0;
        for (int s = 0; s < P; ++s) {
            const uint64_t b = rows[(size_t)s * P + r] * row_bytes;
            recvcounts[(size_t)r * P + s] = b;
            rdispls[(size_t)r * P + s] = run;
            run += b;
        }
    }
    return VCCL_OK;
}

int vccl_plan_alltoallv(void *const *sendbuf, const uint64_t *sendcounts, const uint64_t *sdispls,
                        void *const *recvbuf, const uint64_t *recvcounts, const uint64_t *rdispls, int P,
                        int cu_unroll, int cu_threads, vccl_plan_desc *out, int out_cap, int *n_out,
                        uint32_t *grid_x, uint32_t *grid_y, uint32_t *tile_bytes, int *all_aligned) {
    if (P < 1 || P > VCCL_MAX_RANKS) return fail(VCCL_ERR_ARG, "P = %d is outside 1..%d", P, VCCL_MAX_RANKS);
    if (!sendbuf || !recvbuf || !sendcounts || !sdispls || !recvcounts || !rdispls || !n_out)
        return fail(VCCL_ERR_ARG, "NULL argument");
    if (!(cu_unroll == 1 || cu_unroll == 2 || cu_unroll == 4 || cu_unroll == 8 || cu_unroll == 16))
        return fail(VCCL_ERR_ARG, "cu_unroll must be 1, 2, 4, 8 or 16");
    if (!(cu_threads == 64 || cu_threads == 128 || cu_threads == 256))
        return fail(VCCL_ERR_ARG, "cu_threads must be 64, 128 or 256");
    std::vector<Piece> pieces;
    int rv = alltoallv_pieces(sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P, pieces);
    if (rv) return rv;
    CopyPlan plan;
    for (const Piece &pc : pieces) plan.segs.push_back(Seg{pc.src, pc.dst, pc.bytes, 0, 0});
    rv = plan_tiles(plan, cu_unroll, cu_threads, true);
    if (rv) return rv;
    *n_out = (int)plan.segs.size();
    if (grid_x) *grid_x = plan.max_tiles;
    if (grid_y) *grid_y = (uint32_t)(plan.segs.size() > 65535 ? 65535 : plan.segs.size());
    if (all_aligned) *all_aligned = plan.all_aligned ? 1 : 0;
    if (tile_bytes) *tile_bytes = (uint32_t)(cu_unroll * plan.threads * 16);
    if (out) {
        if ((size_t)out_cap < plan.segs.size())
            return fail(VCCL_ERR_ARG, "the plan has %zu descriptors, room for %d", plan.segs.size(), out_cap);
        for (size_t i = 0; i < plan.segs.size(); ++i) {
            out[i].src = reinterpret_cast<uintptr_t>(plan.segs[i].src);
            out[i].dst = reinterpret_cast<uintptr_t>(plan.segs[i].dst);
            out[i].bytes = plan.segs[i].bytes;
            out[i].head = plan.segs[i].head;
            out[i].lead = plan.segs[i].lead;
        }
    }
    return VCCL_OK;
}

static int fma_probe(float *out_dev, uint64_t *clocks_dev, uint32_t workgroups, uint32_t threads, uint64_t iters,
                     void *stream) {
    auto c = ctx_get();
    if (!c) return fail(VCCL_ERR_NOT_INIT, "vccl_init has not been called");
    if (!out_dev) return fail(VCCL_ERR_ARG, "out_dev is NULL");
    if (threads == 0 || threads > 1024 || (threads & 63u))
        return fail(VCCL_ERR_ARG, "threads = %u must be a multiple of 64 up to 1024", threads);
    if (workgroups == 0) workgroups = (uint32_t)c->cu_count;
    if (workgroups > (1u << 20)) return fail(VCCL_ERR_ARG, "workgroups = %u is too large", workgroups);
    return launch_fma_probe(out_dev, clocks_dev, workgroups, threads, iters, (hipStream_t)stream);
}

int vccl_fma_probe(float *out_dev, uint32_t workgroups, uint32_t threads, uint64_t iters, void *stream) {
    return fma_probe(out_dev, nullptr, workgroups, threads, iters, stream);
}

int vccl_fma_probe_clocks(float *out_dev, uint64_t *clocks_dev, uint32_t workgroups, uint32_t threads,
                          uint64_t iters, void *stream) {
    if (!clocks_dev) return fail(VCCL_ERR_ARG, "clocks_dev is NULL");
    if (reinterpret_cast<uintptr_t>(clocks_dev) & 7u) return fail(VCCL_ERR_ARG, "clocks_dev is not 8-byte aligned");
    return fma_probe(out_dev, clocks_dev, workgroups, threads, iters, stream);
}

int vccl_device_wall_clock_khz(void) {
    auto c = ctx_get();
    if (!c) return fail(VCCL_ERR_NOT_INIT, "vccl_init has not been called");
    int khz = 0;
    VCCL_HIP(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, c->device));
    return khz;
}

int vccl_hbm_probe(int kind, const void *src, void *dst, uint64_t bytes, int threads, int vecs_per_lane,
                   const uint32_t *row_index, uint64_t n_rows, uint64_t row_bytes, void *stream) {
    auto c = ctx_get();
    if (!c) return fail(VCCL_ERR_NOT_INIT, "vccl_init has not been called");
    if (kind < 0 || kind > 3) return fail(VCCL_ERR_ARG, "kind %d is not 0 (read), 1 (write), 2 (copy) or 3 (write rows)", kind);
    if (!dst || ((kind == 0 || kind == 2) && !src)) return fail(VCCL_ERR_ARG, "NULL buffer");
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u)
        return fail(VCCL_ERR_ARG, "buffers are not 16-byte aligned");
    if (kind == 3) {
        if (!n_rows || !row_bytes || (row_bytes & 15u) || (row_bytes >> 4) > 0xffffffffull)
            return fail(VCCL_ERR_ARG, "n_rows = %llu, row_bytes = %llu (a positive multiple of 16)",
                        (unsigned long long)n_rows, (unsigned long long)row_bytes);
    } else if (!bytes || (bytes & 15u)) {
        return fail(VCCL_ERR_ARG, "bytes = %llu must be a positive multiple of 16", (unsigned long long)bytes);
    }
    return launch_hbm_probe(kind, src, dst, bytes, threads, vecs_per_lane, row_index, n_rows, row_bytes,
                            (hipStream_t)stream);
}

int vccl_sendrecv_staged_status(void) {
    auto c = ctx_get();
    if (!c) return fail(VCCL_ERR_NOT_INIT, "vccl_init has not been called");
    uint32_t st = 0;
    int rv = fifo_last_status(c->fifo, &st);
    if (rv) return rv;
    if (st) return fail(VCCL_ERR_TIMEOUT, "a staged SendRecv wait exceeded fifo_spin_limit polls");
    return VCCL_OK;
}

int vccl_proxy_stats(uint64_t *ops, uint64_t *copies, uint64_t *bytes, uint64_t *issue_ns) {
    auto c = ctx_get();
    if (!c) return fail(VCCL_ERR_NOT_INIT, "vccl_init has not been called");
    proxy_stats(c->proxy, ops, copies, bytes, issue_ns);
    return VCCL_OK;
}

int vccl_proxy_cpu_time(uint64_t *sender_ns, uint64_t *receiver_ns) {
    auto c = ctx_get();
    if (!c) return fail(VCCL_ERR_NOT_INIT, "vccl_init has not been called");
    return proxy_cpu_time(c->proxy, sender_ns, receiver_ns);
}

int vccl_proxy_monitor(int primitive, uint64_t *messages, uint64_t *anomalies, vccl_monitor_sample *last) {
    auto c = ctx_get();
    if (!c) return fail(VCCL_ERR_NOT_INIT, "vccl_init has not been called");
    vccl_monitor *m = proxy_monitor(c->proxy, primitive);
    if (!m) return fail(VCCL_ERR_ARG, "primitive must be 0 (SendRecv) or 1 (AlltoAll(v))");
    return vccl_monitor_totals(m, messages, anomalies, last);
}

}  // extern "C"

// ---- SendRecv between two processes (Section 3.2: the receiver's application buffer is
// exported once with an IPC handle and mapped into the sender at connect; the handshake
// record lives in host shared memory; the sender's proxy moves the data with the copy
// engines straight into the receiver's buffer)
struct vccl_p2p_conn {
    int role = 0;                     // 1 sender, 2 receiver
    std::string name;
    P2pShared *sh = nullptr;
    uint8_t *buffer = nullptr;        // receiver: its own buffer; sender: the same memory as mapped here
    void *mapped_alloc = nullptr;     // sender: what hipIpcOpenMemHandle returned
    uint64_t next_seq = 0;            // transfers posted so far on this side
    std::mutex mu;
};

static int p2p_name_ok(const char *name) {
    if (!name || name[0] != '/' || strlen(name) < 2 || strlen(name) > 200 || strchr(name + 1, '/'))
        return fail(VCCL_ERR_ARG, "a connection name is '/' followed by 1..199 characters without '/'");
    return VCCL_OK;
}

extern "C" {

int vccl_p2p_export(const char *name, void *recvbuf_dev, uint64_t capacity, vccl_p2p_conn **out) {
    auto c = ctx_get();
    if (!c) return fail(VCCL_ERR_NOT_INIT, "vccl_init has not been called");
    int rv = p2p_name_ok(name);
    if (rv) return rv;
    if (!recvbuf_dev || !capacity || !out) return fail(VCCL_ERR_ARG, "NULL buffer, zero capacity or NULL out");
    // The handle names the whole allocation the buffer lies in; the record carries the offset.
    void *base = nullptr;
    size_t alloc_size = 0;
    VCCL_HIP(hipMemGetAddressRange((hipDeviceptr_t *)&base, &alloc_size, (hipDeviceptr_t)recvbuf_dev));
    const uint64_t off = (uint64_t)((uint8_t *)recvbuf_dev - (uint8_t *)base);
    if (off + capacity > alloc_size)
        return fail(VCCL_ERR_ARG, "the buffer (+%llu, %llu bytes) does not lie inside one allocation of %zu bytes",
                    (unsigned long long)off, (unsigned long long)capacity, alloc_size);
    if (alloc_size >= (2ull << 30))
        return fail(VCCL_ERR_UNSUPPORTED, "the allocation holding the buffer has %zu bytes; allocations shared "
                                          "between processes must stay below 2 GiB", alloc_size);
    hipIpcMemHandle_t h;
    static_assert(sizeof(h) <= sizeof(P2pShared::ipc_handle), "handle size");
    VCCL_HIP(hipIpcGetMemHandle(&h, base));
    const int fd = shm_open(name, O_CREAT | O_EXCL | O_RDWR, 0600);
    if (fd < 0) return fail(VCCL_ERR_ARG, "shm_open(%s) failed: %s", name, strerror(errno));
    if (ftruncate(fd, (off_t)sizeof(P2pShared)) != 0) {
        const int e = errno;
        close(fd);
        shm_unlink(name);
        return fail(VCCL_ERR_ARG, "ftruncate(%s) failed: %s", name, strerror(e));
    }
    void *m = mmap(nullptr, sizeof(P2pShared), PROT_READ | PROT_WRITE, MAP_SHARED, fd, 0);
    close(fd);
    if (m == MAP_FAILED) {
        shm_unlink(name);
        return fail(VCCL_ERR_ARG, "mmap(%s) failed", name);
    }
    P2pShared *sh = new (m) P2pShared();      // a fresh object in zero-filled pages
    sh->capacity = capacity;
    sh->alloc_offset = off;
    sh->receiver_pid = (int32_t)getpid();
    memcpy(sh->ipc_handle, &h, sizeof(h));
    std::atomic_thread_fence(std::memory_order_release);
    reinterpret_cast<std::atomic<uint64_t> *>(&sh->magic)->store(kP2pMagic, std::memory_order_release);
    vccl_p2p_conn *conn = new vccl_p2p_conn;
    conn->role = 2;
    conn->name = name;
    conn->sh = sh;
    conn->buffer = (uint8_t *)recvbuf_dev;
    *out = conn;
    return VCCL_OK;
}

int vccl_p2p_connect(const char *name, double timeout_s, vccl_p2p_conn **out) {
    auto c = ctx_get();
    if (!c) return fail(VCCL_ERR_NOT_INIT, "vccl_init has not been called");
    int rv = p2p_name_ok(name);
    if (rv) return rv;
    if (!out) return fail(VCCL_ERR_ARG, "NULL out");
    struct timespec t0;
    clock_gettime(CLOCK_MONOTONIC, &t0);
    auto waited = [&] {
        struct timespec t;
        clock_gettime(CLOCK_MONOTONIC, &t);
        return (double)(t.tv_sec - t0.tv_sec) + 1e-9 * (double)(t.tv_nsec - t0.tv_nsec);
    };
    P2pShared *sh = nullptr;
    for (;;) {   // the receiver may not have exported yet
        const int fd = shm_open(name, O_RDWR, 0600);
        if (fd >= 0) {
            struct stat st;
            if (fstat(fd, &st) == 0 && (size_t)st.st_size >= sizeof(P2pShared)) {
                void *m = mmap(nullptr, sizeof(P2pShared), PROT_READ | PROT_WRITE, MAP_SHARED, fd, 0);
                if (m != MAP_FAILED) {
                    sh = static_cast<P2pShared *>(m);
                    if (reinterpret_cast<std::atomic<uint64_t> *>(&sh->magic)->load(std::memory_order_acquire) ==
                        kP2pMagic) {
                        close(fd);
                        break;
                    }
                    munmap(m, sizeof(P2pShared));
                    sh = nullptr;
                }
            }
            close(fd);
        }
        if (waited() > timeout_s) return fail(VCCL_ERR_TIMEOUT, "no exported connection '%s' after %.1f s", name, timeout_s);
        usleep(2000);
    }
    if (sh->sender_attached.exchange(1) != 0) {
        munmap(sh, sizeof(P2pShared));
        return fail(VCCL_ERR_ARG, "connection '%s' already has a sender", name);
    }
    // a handle whose exporting process is gone must not be opened
    if (sh->receiver_closed.load() || sh->aborted.load() || (kill((pid_t)sh->receiver_pid, 0) != 0 && errno == ESRCH)) {
        sh->sender_attached.store(0);
        munmap(sh, sizeof(P2pShared));
        return fail(VCCL_ERR_ARG, "the receiver of connection '%s' is gone", name);
    }
    hipIpcMemHandle_t h;
    memcpy(&h, sh->ipc_handle, sizeof(h));
    void *mapped = nullptr;
    hipError_t e = hipIpcOpenMemHandle(&mapped, h, hipIpcMemLazyEnablePeerAccess);
    if (e != hipSuccess) {
        sh->sender_attached.store(0);
        munmap(sh, sizeof(P2pShared));
        return fail(VCCL_ERR_HIP, "hipIpcOpenMemHandle failed: %s", hipGetErrorString(e));
    }
    vccl_p2p_conn *conn = new vccl_p2p_conn;
    conn->role = 1;
    conn->name = name;
    conn->sh = sh;
    conn->mapped_alloc = mapped;
    conn->buffer = (uint8_t *)mapped + sh->alloc_offset;
    *out = conn;
    return VCCL_OK;
}

int vccl_p2p_recv(vccl_p2p_conn *conn, uint64_t offset, uint64_t bytes, void *stream) {
    auto c = ctx_get();
    if (!c) return fail(VCCL_ERR_NOT_INIT, "vccl_init has not been called");
    if (!conn || conn->role != 2) return fail(VCCL_ERR_ARG, "not the receiving end of a connection");
    if (conn->sh->aborted.load()) return fail(VCCL_ERR_TIMEOUT, "connection '%s' was aborted", conn->name.c_str());
    if (offset > conn->sh->capacity || bytes > conn->sh->capacity - offset)
        return fail(VCCL_ERR_ARG, "offset %llu + %llu bytes exceed the registered %llu", (unsigned long long)offset,
                    (unsigned long long)bytes, (unsigned long long)conn->sh->capacity);
    std::lock_guard<std::mutex> lk(conn->mu);   // posts of one connection reach the proxy in sequence order
    const uint64_t seq = conn->next_seq + 1;
    int rv = proxy_submit_remote(c->proxy, 2, conn->sh, nullptr, seq, nullptr, offset, bytes, options_of(*c),
                                 (hipStream_t)stream);
    if (rv == VCCL_OK) conn->next_seq = seq;
    return rv;
}

int vccl_p2p_send(vccl_p2p_conn *conn, const void *sendbuf_dev, uint64_t bytes, void *stream) {
    auto c = ctx_get();
    if (!c) return fail(VCCL_ERR_NOT_INIT, "vccl_init has not been called");
    if (!conn || conn->role != 1) return fail(VCCL_ERR_ARG, "not the sending end of a connection");
    if (bytes && !sendbuf_dev) return fail(VCCL_ERR_ARG, "NULL send buffer");
    if (conn->sh->aborted.load()) return fail(VCCL_ERR_TIMEOUT, "connection '%s' was aborted", conn->name.c_str());
    std::lock_guard<std::mutex> lk(conn->mu);
    const uint64_t seq = conn->next_seq + 1;
    int rv = proxy_submit_remote(c->proxy, 1, conn->sh, conn->buffer, seq, sendbuf_dev, 0, bytes, options_of(*c),
                                 (hipStream_t)stream);
    if (rv == VCCL_OK) conn->next_seq = seq;
    return rv;
}

int vccl_p2p_record(vccl_p2p_conn *conn, uint64_t *receiver_ready, uint64_t *copy_started, uint64_t *copy_done,
                    uint64_t *reg_offset, uint64_t *mismatches) {
    if (!conn || !conn->sh) return fail(VCCL_ERR_ARG, "NULL connection");
    const P2pShared *sh = conn->sh;
    if (receiver_ready) *receiver_ready = sh->receiverReady.load(std::memory_order_acquire);
    if (copy_started) *copy_started = sh->copyStarted.load(std::memory_order_acquire);
    if (copy_done) *copy_done = sh->copyDone.load(std::memory_order_acquire);
    if (reg_offset) *reg_offset = sh->receiverRegOffset.load(std::memory_order_acquire);
    if (mismatches) *mismatches = sh->mismatches.load(std::memory_order_acquire);
    return VCCL_OK;
}

int vccl_p2p_abort(vccl_p2p_conn *conn) {
    if (!conn || !conn->sh) return fail(VCCL_ERR_ARG, "NULL connection");
    conn->sh->aborted.store(1, std::memory_order_release);
    return VCCL_OK;
}

int vccl_p2p_close(vccl_p2p_conn *conn) {
    if (!conn) return fail(VCCL_ERR_ARG, "NULL connection");
    auto c = ctx_get();
    int rv = VCCL_OK;
    // No operation of this process may still point at the record when it is unmapped.  A
    // transfer whose other side never comes would wait for ever: after the deadline the
    // connection is aborted, which ends every outstanding transfer at the proxy's next poll.
    if (c && !proxy_drain_for(c->proxy, 1e-3 * options_of(*c).p2p_close_wait_ms) &&
        conn->sh->copyDone.load(std::memory_order_acquire) < conn->next_seq) {
        conn->sh->aborted.store(1, std::memory_order_release);
        rv = fail(VCCL_ERR_TIMEOUT, "connection '%s' closed with transfers outstanding: aborted", conn->name.c_str());
        if (!proxy_drain_for(c->proxy, 10.0)) return rv;   // an aborted transfer ends at the next poll; something else holds the proxy up: keep the mappings
    }
    if (conn->role == 1) {
        if (conn->mapped_alloc && hipIpcCloseMemHandle(conn->mapped_alloc) != hipSuccess && rv == VCCL_OK)
            rv = fail(VCCL_ERR_HIP, "hipIpcCloseMemHandle failed");
        conn->sh->sender_attached.store(0);
    } else {
        conn->sh->receiver_closed.store(1);
        shm_unlink(conn->name.c_str());
    }
    munmap(conn->sh, sizeof(P2pShared));
    delete conn;
    return rv;
}

int vccl_p2p_reginfo(int receiver_rank, uint64_t *receiver_ready, uint64_t *copy_started,
                     uint64_t *copy_done, void **receiver_reg_addr) {
    auto c = ctx_get();
    if (!c) return fail(VCCL_ERR_NOT_INIT, "vccl_init has not been called");
    return proxy_reginfo(c->proxy, receiver_rank, receiver_ready, copy_started, copy_done,
                         receiver_reg_addr);
}

}  // extern "C"
