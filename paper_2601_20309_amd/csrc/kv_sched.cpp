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

int kv_sched_lvf(const kv_sched_params *p, const kv_sched_req *reqs, int32_t n, double t_now, int32_t b_xfer,
                 int32_t b_hbm, int32_t *preempt, int32_t *n_preempt, int32_t *prioritize, int32_t *n_prioritize,
                 int32_t *fcfs)
{
    if (!p || n < 0 || (n > 0 && !reqs) || b_xfer < 0 || b_hbm < 0 || !n_preempt || !n_prioritize ||
        (n > 0 && (!preempt || !prioritize)))
        return KV_EINVAL;
    int64_t inactive_blocks = 0;
    for (int32_t i = 0; i < n; i++) {
        if (reqs[i].state < KV_REQ_RUNNING || reqs[i].state > KV_REQ_ROTARY || reqs[i].blocks < 0) return KV_EINVAL;
        if (reqs[i].state != KV_REQ_RUNNING) inactive_blocks += reqs[i].blocks;
    }
    *n_preempt = *n_prioritize = 0;
    if (fcfs) *fcfs = 0;
    std::vector<int32_t> order((size_t)n);
    for (int32_t i = 0; i < n; i++) order[(size_t)i] = i;
    if ((int64_t)b_hbm >= inactive_blocks) {  // no contention: first come first served
        std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
            return reqs[a].t_ref != reqs[b].t_ref ? reqs[a].t_ref < reqs[b].t_ref : reqs[a].id < reqs[b].id;
        });
        for (int32_t k : order)
            if (reqs[k].state != KV_REQ_RUNNING) prioritize[(*n_prioritize)++] = reqs[k].id;
        if (fcfs) *fcfs = 1;
        return KV_OK;
    }
    std::vector<double> vlt((size_t)n);
    for (int32_t i = 0; i < n; i++) vlt[(size_t)i] = kv_sched_vlt(p, &reqs[i], t_now);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        return vlt[(size_t)a] != vlt[(size_t)b] ? vlt[(size_t)a] > vlt[(size_t)b] : reqs[a].id < reqs[b].id;
    });
    int64_t left = (int64_t)b_hbm + b_xfer;
    for (int32_t k : order) {
        if (reqs[k].state != KV_REQ_RUNNING && vlt[(size_t)k] >= 0.0 && reqs[k].blocks <= left) {
            prioritize[(*n_prioritize)++] = reqs[k].id;
            left -= reqs[k].blocks;
        }
    }
    int64_t swap = (int64_t)b_xfer - left;
    for (auto it = order.rbegin(); it != order.rend() && swap > 0; ++it) {
        const int32_t k = *it;
        if (reqs[k].state == KV_REQ_RUNNING && vlt[(size_t)k] < 0.0) {
            preempt[(*n_preempt)++] = reqs[k].id;
            swap -= reqs[k].blocks;
        }
    }
    return KV_OK;
}

}  // extern "C"
