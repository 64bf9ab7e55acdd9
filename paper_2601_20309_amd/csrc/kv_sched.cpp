// Virtual Lag Time and Largest-VLT-First scheduling (paper Section 4.2.1, the
// VLT equation, and Section 4.2.2, Algorithm 1).  Plain host C++, no HIP.
#include <algorithm>
#include <cstdint>
#include <vector>

#include "../../include/duplexkv.h"

extern "C" {

double kv_sched_vlt(const kv_sched_params *p, const kv_sched_req *r, double t_now)
{
    if (!p || !r) return 0.0;
    const double idle = t_now - r->t_ref;
    switch (r->state) {
    case KV_REQ_ROTARY: return p->alpha * std::max(0.0, idle - p->beta_b * p->slo_tbt);
    case KV_REQ_WAITING: return std::max(0.0, idle - p->beta_f * p->slo_ttft);
    default: return -idle;
    }
}

}  // extern "C"

namespace {

// One request as the selection sees it: its lag, and where it stood in the input
// (the last tie-break, so that the outcome never depends on the sort routine).
struct Entry {
    double key;  // VLT, or the reference time for first come first served
    int32_t id, blocks, at;
};

// "Comes earlier in the queue sorted by VLT, largest first; ties: smaller id."
bool ahead(const Entry &a, const Entry &b)
{
    if (a.key != b.key) return a.key > b.key;
    if (a.id != b.id) return a.id < b.id;
    return a.at < b.at;
}

}  // namespace

extern "C" {

// Algorithm 1 of the paper walks one queue sorted by VLT twice, from the head for
// the requests to bring in and from the tail for the requests to push out.  Only
// waiting / rotary requests are ever taken from the head and only running ones
// from the tail, so the two walks are done here on the two groups separately:
// the inactive group is sorted and filled greedily into b_hbm + b_xfer blocks;
// the running group is a heap keyed the other way round, from which victims are
// popped only as long as the blocks granted exceed what is free.
int kv_sched_lvf(const kv_sched_params *p, const kv_sched_req *reqs, int32_t n, double t_now, int32_t b_xfer,
                 int32_t b_hbm, int32_t *preempt, int32_t *n_preempt, int32_t *prioritize, int32_t *n_prioritize,
                 int32_t *fcfs)
{
    if (!p || n < 0 || (n > 0 && !reqs) || b_xfer < 0 || b_hbm < 0 || !n_preempt || !n_prioritize ||
        (n > 0 && (!preempt || !prioritize)))
        return KV_EINVAL;
    std::vector<Entry> inactive, running;
    int64_t inactive_blocks = 0;
    for (int32_t i = 0; i < n; i++) {
        const kv_sched_req &r = reqs[i];
        if (r.state < KV_REQ_RUNNING || r.state > KV_REQ_ROTARY || r.blocks < 0) return KV_EINVAL;
        (r.state == KV_REQ_RUNNING ? running : inactive).push_back(Entry{0.0, r.id, r.blocks, i});
        if (r.state != KV_REQ_RUNNING) inactive_blocks += r.blocks;
    }
    int32_t n_pri = 0, n_pre = 0;
    *n_preempt = *n_prioritize = 0;
    if (fcfs) *fcfs = 0;
    if (inactive_blocks <= (int64_t)b_hbm) {
        // no contention: everybody comes in, oldest reference time first
        for (Entry &e : inactive) e.key = -reqs[e.at].t_ref;
        std::sort(inactive.begin(), inactive.end(), ahead);
        for (const Entry &e : inactive) prioritize[n_pri++] = e.id;
        *n_prioritize = n_pri;
        if (fcfs) *fcfs = 1;
        return KV_OK;
    }
    for (Entry &e : inactive) e.key = kv_sched_vlt(p, &reqs[e.at], t_now);
    std::sort(inactive.begin(), inactive.end(), ahead);
    const int64_t room = (int64_t)b_hbm + b_xfer;
    int64_t granted = 0;
    for (const Entry &e : inactive) {
        if (e.key >= 0.0 && granted + e.blocks <= room) {
            prioritize[n_pri++] = e.id;
            granted += e.blocks;
        }
    }
    // blocks that have to be freed: what was granted beyond the free ones
    int64_t owed = granted - (int64_t)b_hbm;
    if (owed > 0) {
        size_t m = 0;
        for (const Entry &e : running) {
            const double v = kv_sched_vlt(p, &reqs[e.at], t_now);
            if (v < 0.0) running[m++] = Entry{v, e.id, e.blocks, e.at};
        }
        running.resize(m);
        // max-heap under `ahead`: the top is the request that comes LAST in the queue
        auto last_first = [](const Entry &a, const Entry &b) { return ahead(a, b); };
        std::make_heap(running.begin(), running.end(), last_first);
        while (owed > 0 && !running.empty()) {
            std::pop_heap(running.begin(), running.end(), last_first);
            const Entry v = running.back();
            running.pop_back();
            preempt[n_pre++] = v.id;
            owed -= v.blocks;
        }
    }
    *n_prioritize = n_pri;
    *n_preempt = n_pre;
    return KV_OK;
}

}  // extern "C"
