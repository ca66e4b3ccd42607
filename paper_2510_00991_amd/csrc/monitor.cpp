// Window-based bandwidth monitor (paper Section 3.4), applied here to the copies
// the proxy issues instead of RDMA work requests: a message is posted at t1 and
// completes at t2; the per-message estimate is bytes / (t2 - t1); the window
// estimate divides the bytes of the last `window` completed messages by the span
// from the earliest post to the latest completion among them (window 8 in the
// paper's deployment).  A completion is flagged as an anomaly when its window
// estimate is below half the mean estimate of the preceding history span AND the
// outstanding (posted, not completed) bytes exceed twice the largest outstanding
// amount seen in that span.  The span is the `history` nanoseconds that end where
// the current window begins, so the messages being judged do not vote on their
// own baseline.  Pure host code: no device is needed.
#include <deque>
#include <mutex>
#include <unordered_map>

#include "common.h"

struct vccl_monitor {
    int window;
    uint64_t history_ns;
    std::mutex mu;
    struct Msg {
        uint64_t post, done, bytes;
    };
    struct Past {
        uint64_t t;
        double bw;
        uint64_t outstanding;
    };
    std::unordered_map<uint64_t, Msg> in_flight;
    std::deque<Msg> recent;      // last `window` completed messages, completion order
    std::deque<Past> past;       // earlier evaluations, time order
    uint64_t outstanding = 0;
    uint64_t messages = 0, anomalies = 0;
    vccl_monitor_sample last = {};
};

extern "C" {

vccl_monitor *vccl_monitor_create(int window, uint64_t history_ns) {
    if (window < 1 || window > 65536 || history_ns == 0) {
        vccl::fail(VCCL_ERR_ARG, "monitor window %d / history %llu ns out of range", window,
                   (unsigned long long)history_ns);
        return nullptr;
    }
    vccl_monitor *m = new vccl_monitor;
    m->window = window;
    m->history_ns = history_ns;
    return m;
}

void vccl_monitor_destroy(vccl_monitor *m) { delete m; }

int vccl_monitor_post(vccl_monitor *m, uint64_t id, uint64_t bytes, uint64_t t_post_ns) {
    if (!m) return vccl::fail(VCCL_ERR_ARG, "NULL monitor");
    std::lock_guard<std::mutex> lk(m->mu);
    if (!m->in_flight.emplace(id, vccl_monitor::Msg{t_post_ns, 0, bytes}).second)
        return vccl::fail(VCCL_ERR_ARG, "message id %llu is already in flight", (unsigned long long)id);
    m->outstanding += bytes;
    return VCCL_OK;
}

int vccl_monitor_complete(vccl_monitor *m, uint64_t id, uint64_t t_done_ns, vccl_monitor_sample *out) {
    if (!m) return vccl::fail(VCCL_ERR_ARG, "NULL monitor");
    std::lock_guard<std::mutex> lk(m->mu);
    auto it = m->in_flight.find(id);
    if (it == m->in_flight.end())
        return vccl::fail(VCCL_ERR_ARG, "message id %llu was not posted", (unsigned long long)id);
    vccl_monitor::Msg msg = it->second;
    m->in_flight.erase(it);
    if (t_done_ns <= msg.post)
        return vccl::fail(VCCL_ERR_ARG, "completion time must be later than the post time");
    msg.done = t_done_ns;
    m->outstanding -= msg.bytes;
    m->recent.push_back(msg);
    if ((int)m->recent.size() > m->window) m->recent.pop_front();
    uint64_t t1 = ~0ull, t2 = 0, sum = 0;
    for (const auto &r : m->recent) {
        if (r.post < t1) t1 = r.post;
        if (r.done > t2) t2 = r.done;
        sum += r.bytes;
    }
    vccl_monitor_sample s;
    s.t_ns = t_done_ns;
    s.bw_message = (double)msg.bytes / ((double)(t_done_ns - msg.post) * 1e-9);
    s.bw_window = (double)sum / ((double)(t2 - t1) * 1e-9);
    s.outstanding = m->outstanding;
    // baseline: evaluations inside [t1 - history, t1)
    const uint64_t lo = t1 > m->history_ns ? t1 - m->history_ns : 0;
    double acc = 0.0;
    uint64_t n = 0, peak = 0;
    for (const auto &p : m->past) {
        if (p.t < lo || p.t >= t1) continue;
        acc += p.bw;
        ++n;
        if (p.outstanding > peak) peak = p.outstanding;
    }
    s.anomaly = (n > 0 && s.bw_window < 0.5 * (acc / (double)n) && s.outstanding > 2 * peak) ? 1 : 0;
    m->past.push_back(vccl_monitor::Past{t_done_ns, s.bw_window, s.outstanding});
    // No later window can begin before the earliest post among the messages still in
    // flight or in the current window; evaluations older than one history span
    // before that can never be consulted again.
    uint64_t earliest = t1;
    for (const auto &kv : m->in_flight)
        if (kv.second.post < earliest) earliest = kv.second.post;
    const uint64_t keep_from = earliest > m->history_ns ? earliest - m->history_ns : 0;
    while (!m->past.empty() && m->past.front().t < keep_from) m->past.pop_front();
    ++m->messages;
    m->anomalies += (uint64_t)s.anomaly;
    m->last = s;
    if (out) *out = s;
    return VCCL_OK;
}

int vccl_monitor_totals(vccl_monitor *m, uint64_t *messages, uint64_t *anomalies, vccl_monitor_sample *last) {
    if (!m) return vccl::fail(VCCL_ERR_ARG, "NULL monitor");
    std::lock_guard<std::mutex> lk(m->mu);
    if (messages) *messages = m->messages;
    if (anomalies) *anomalies = m->anomalies;
    if (last) *last = m->last;
    return VCCL_OK;
}

}  // extern "C"
