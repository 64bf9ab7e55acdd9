// Block table with eager block rotation on top of the engine (paper Section
// 4.3.2): allocation of HBM blocks and host slots, per-block state, and the
// translation of "these requests leave, those come back" into one duplex
// transfer.  Host code only; every byte is moved by the engine's paths.
#include <algorithm>
#include <cstdint>
#include <new>
#include <utility>
#include <vector>

#include "kv_engine.hpp"

using dkv::list_bad;

namespace {

struct TableReq {
    bool used = false, resident = false;
    int32_t len = 0;
    int32_t n_full = 0;  // blocks in state FULL (filled, copy to DRAM not yet issued)
    // the engine's idle_epoch when a transfer last named HBM blocks of this request
    // (an eager copy that reads them, a resumption that writes them); -1: never
    int64_t named_at = -1;
    std::vector<int32_t> hbm, slot, state;
};

// A set of ids read lowest first: the free blocks, the free slots, the requests
// that have FULL blocks.  One bit per id, plus one bit per 64-id word that says
// "this word has a member", so that the lowest member is two scans of a few
// words (a 288 GB cache of 2 MiB blocks is 2200 words and 35 summary words).
// While a journal is open every change is noted and can be taken back, which is
// how a rotation the engine refuses is undone without copying the set.
class IdSet {
  public:
    void reset(int32_t n)
    {
        bits_.assign(((size_t)n + 63) / 64, 0);
        any_.assign((bits_.size() + 63) / 64, 0);
        count_ = 0;
        journal_.clear();
        open_ = false;
    }
    size_t size() const { return count_; }
    bool empty() const { return count_ == 0; }
    void push(int32_t id) { flip(id, true); }
    void remove(int32_t id) { flip(id, false); }
    // lowest member, -1 if there is none
    int32_t top() const { return next(0); }
    // lowest member >= from, -1 if there is none
    int32_t next(int32_t from) const
    {
        size_t w = (size_t)from / 64;
        if (w >= bits_.size()) return -1;
        const uint64_t here = bits_[w] & (~0ull << ((size_t)from % 64));
        if (here) return (int32_t)(w * 64 + (size_t)__builtin_ctzll(here));
        // the words behind w: the summary bits say which of them have members
        for (size_t nw = w + 1; nw < bits_.size();) {
            const size_t a = nw / 64;
            const uint64_t m = any_[a] & (~0ull << (nw % 64));
            if (m) {
                w = a * 64 + (size_t)__builtin_ctzll(m);
                return (int32_t)(w * 64 + (size_t)__builtin_ctzll(bits_[w]));
            }
            nw = (a + 1) * 64;
        }
        return -1;
    }
    void pop()
    {
        if (count_ > 0) flip(top(), false);
    }
    void open_journal()
    {
        journal_.clear();
        open_ = true;
    }
    // keep = false: every change since open_journal() is taken back, latest first
    void close_journal(bool keep)
    {
        open_ = false;
        if (!keep)
            for (size_t k = journal_.size(); k-- > 0;) flip(journal_[k].first, !journal_[k].second);
        journal_.clear();
    }

  private:
    void flip(int32_t id, bool to_member)
    {
        const size_t w = (size_t)id / 64;
        const uint64_t m = 1ull << ((size_t)id % 64);
        if (to_member == ((bits_[w] & m) != 0)) return;  // already so
        if (to_member) {
            bits_[w] |= m;
            any_[w / 64] |= 1ull << (w % 64);
            count_++;
        } else {
            bits_[w] &= ~m;
            if (!bits_[w]) any_[w / 64] &= ~(1ull << (w % 64));
            count_--;
        }
        if (open_) journal_.emplace_back(id, to_member);
    }
    std::vector<uint64_t> bits_, any_;
    size_t count_ = 0;
    std::vector<std::pair<int32_t, bool>> journal_;  // (id, became a member)
    bool open_ = false;
};

}  // namespace

struct kv_table {
    kv_engine *e = nullptr;
    int32_t max_req = 0;
    std::vector<TableReq> req;
    IdSet free_hbm, free_slot;
    IdSet with_full;  // requests (resident ones) that have blocks in state FULL: the eager step's work list
    kv_table_counts cnt{};
    std::vector<int32_t> oi, os, ii, is, held, seen;
    // What a rotation had before it started, kept until its transfer is accepted:
    // the counters and every request the call changes (the free sets keep a journal).
    kv_table_counts undo_cnt{};
    std::vector<std::pair<int32_t, TableReq>> undo_req;
    std::vector<int32_t> saved;  // per request: 1 if already in undo_req
};

namespace {

void save_request(kv_table *t, int32_t q)
{
    if (t->saved[(size_t)q]) return;
    t->saved[(size_t)q] = 1;
    t->undo_req.emplace_back(q, t->req[(size_t)q]);
}

void begin_undo(kv_table *t)
{
    t->free_hbm.open_journal();
    t->free_slot.open_journal();
    t->with_full.open_journal();
    t->undo_cnt = t->cnt;
    t->undo_req.clear();
}

// ok: forget the saved state; else put everything back as it was.
void end_undo(kv_table *t, bool ok)
{
    for (auto &pr : t->undo_req) {
        t->saved[(size_t)pr.first] = 0;
        if (!ok) t->req[(size_t)pr.first] = std::move(pr.second);
    }
    t->undo_req.clear();
    t->free_hbm.close_journal(ok);
    t->free_slot.close_journal(ok);
    t->with_full.close_journal(ok);
    if (!ok) t->cnt = t->undo_cnt;
}

}  // namespace

extern "C" {

int kv_table_create(kv_table **out, kv_engine *e, int32_t max_requests)
{
    if (!out) return KV_EINVAL;
    *out = nullptr;
    if (!e || max_requests <= 0) return KV_EINVAL;
    if (e->cfg.path == KV_PATH_SDMA_STAGED || e->cfg.path == KV_PATH_NAIVE || e->cfg.path == KV_PATH_DMA_BLOCKS)
        return KV_EUNSUP;
    kv_table *t = new (std::nothrow) kv_table;
    if (!t) return KV_ENOMEM;
    t->e = e;
    t->max_req = max_requests;
    t->req.resize((size_t)max_requests);
    t->free_hbm.reset(e->cfg.n_hbm_blocks);
    t->free_slot.reset(e->cfg.n_host_slots);
    t->with_full.reset(max_requests);
    for (int32_t i = 0; i < e->cfg.n_hbm_blocks; i++) t->free_hbm.push(i);
    for (int32_t i = 0; i < e->cfg.n_host_slots; i++) t->free_slot.push(i);
    t->seen.assign((size_t)max_requests, 0);
    t->saved.assign((size_t)max_requests, 0);
    e->in_after_out = true;
    e->n_tables++;
    *out = t;
    return KV_OK;
}

int kv_table_destroy(kv_table *t)
{
    if (!t) return KV_EINVAL;
    if (--t->e->n_tables == 0) t->e->in_after_out = false;
    delete t;
    return KV_OK;
}

int kv_table_append(kv_table *t, int32_t rq, int32_t n_tokens, int32_t *new_ids, int32_t cap, int32_t *n_new)
{
    if (!t || rq < 0 || rq >= t->max_req || n_tokens < 0) return KV_EINVAL;
    TableReq &r = t->req[(size_t)rq];
    if (r.used && !r.resident) return KV_EINVAL;
    const int32_t P = t->e->cfg.block_size;
    const int32_t old_len = r.used ? r.len : 0, old_n = r.used ? (int32_t)r.hbm.size() : 0;
    const int64_t new_len = (int64_t)old_len + n_tokens;
    const int64_t need = (new_len + P - 1) / P - old_n;
    if (need > (int64_t)t->free_hbm.size()) return KV_ENOSPC;
    if (new_ids && need > cap) return KV_EINVAL;
    if (!r.used) {
        r = TableReq{};
        r.used = r.resident = true;
    }
    if (n_tokens > 0 && old_len % P != 0) r.state[(size_t)old_n - 1] = KV_BLOCK_DIRTY;
    for (int64_t k = 0; k < need; k++) {
        const int32_t b = t->free_hbm.top();
        t->free_hbm.pop();
        r.hbm.push_back(b);
        r.slot.push_back(-1);
        r.state.push_back(KV_BLOCK_DIRTY);
        if (new_ids) new_ids[k] = b;
    }
    r.len = (int32_t)new_len;
    // blocks that this call filled up: the former tail and the new ones, but for the new tail
    for (size_t i = old_n > 0 ? (size_t)old_n - 1 : 0; i < r.hbm.size(); i++) {
        if ((int64_t)(i + 1) * P <= r.len && r.state[i] == KV_BLOCK_DIRTY) {
            r.state[i] = KV_BLOCK_FULL;
            r.n_full++;
        }
    }
    if (r.n_full > 0) t->with_full.push(rq);
    if (n_new) *n_new = (int32_t)need;
    return KV_OK;
}

// Eager step's choice: up to `budget` FULL blocks of resident requests, by
// request id, then block index; each gets a slot (its own, else the lowest free
// one) and is appended to the out list.  Stops when the pool is exhausted.
static void pick_eager(kv_table *t, int32_t budget, std::vector<std::pair<int32_t, size_t>> &picked,
                       std::vector<int32_t> &fresh)
{
    int32_t n = 0;
    for (int32_t q = t->with_full.top(); q >= 0 && n < budget; q = t->with_full.next(q + 1)) {
        TableReq &r = t->req[(size_t)q];
        for (size_t i = 0; i < r.hbm.size() && n < budget; i++) {
            if (r.state[i] != KV_BLOCK_FULL) continue;
            int32_t sl = r.slot[i];
            if (sl < 0) {
                if (t->free_slot.empty()) return;
                sl = t->free_slot.top();
                t->free_slot.pop();
                fresh.push_back(sl);
            }
            t->oi.push_back(r.hbm[i]);
            t->os.push_back(sl);
            picked.push_back({q, i});
            n++;
        }
    }
}

static void mark_synced(kv_table *t, const std::vector<std::pair<int32_t, size_t>> &picked, size_t first,
                        bool undoable = false)
{
    for (size_t k = 0; k < picked.size(); k++) {
        if (undoable) save_request(t, picked[k].first);
        TableReq &r = t->req[(size_t)picked[k].first];
        r.slot[picked[k].second] = t->os[first + k];
        r.state[picked[k].second] = KV_BLOCK_SYNCED;
        if (--r.n_full == 0) t->with_full.remove(picked[k].first);
    }
}

int kv_table_eager(kv_table *t, int32_t budget, int32_t *n_done)
{
    if (!t || budget < 0) return KV_EINVAL;
    t->oi.clear();
    t->os.clear();
    std::vector<std::pair<int32_t, size_t>> picked;  // (request, block index)
    std::vector<int32_t> fresh;                      // slots taken for this call
    pick_eager(t, budget, picked, fresh);
    if (!t->oi.empty()) {
        int rc = kv_swap_out(t->e, t->oi.data(), t->os.data(), (int32_t)t->oi.size());
        if (rc != KV_OK) {
            for (int32_t sl : fresh) t->free_slot.push(sl);
            return rc;
        }
        mark_synced(t, picked, 0);
        for (const auto &pk : picked) t->req[(size_t)pk.first].named_at = (int64_t)t->e->idle_epoch;
    }
    t->cnt.copied_eager += (int64_t)t->oi.size();
    if (n_done) *n_done = (int32_t)t->oi.size();
    return KV_OK;
}

// Are the named requests known, named once, and where the call needs them
// (resident to leave, in DRAM to come back)?
static bool names_ok(kv_table *t, const int32_t *pre, int32_t n_pre, const int32_t *res, int32_t n_res)
{
    bool ok = true;
    auto claim = [&](int32_t q, bool want_resident) {
        if (q < 0 || q >= t->max_req) return false;
        const TableReq &r = t->req[(size_t)q];
        if (!r.used || r.resident != want_resident || t->seen[(size_t)q]) return false;
        t->seen[(size_t)q] = 1;
        return true;
    };
    int32_t marked_pre = 0, marked_res = 0;  // entries claimed so far
    while (ok && marked_pre < n_pre) {
        ok = claim(pre[marked_pre], true);
        if (ok) marked_pre++;
    }
    while (ok && marked_res < n_res) {
        ok = claim(res[marked_res], false);
        if (ok) marked_res++;
    }
    for (int32_t i = 0; i < marked_pre; i++) t->seen[(size_t)pre[i]] = 0;
    for (int32_t i = 0; i < marked_res; i++) t->seen[(size_t)res[i]] = 0;
    return ok;
}

// A request leaves HBM.  Blocks with a valid DRAM copy are released on the spot,
// without a byte moving, and may be refilled by this very call; the others join
// the out list (taking the lowest free slot if they have none) and stay out of
// the free set until the call's swap-ins have been placed, because a block this
// call still reads must not be one it writes.  False: the pool has no slot left.
static bool leave_hbm(kv_table *t, int32_t q, int64_t &released)
{
    save_request(t, q);
    TableReq &r = t->req[(size_t)q];
    for (size_t b = 0; b < r.hbm.size(); b++) {
        const int32_t id = r.hbm[b];
        if (r.state[b] == KV_BLOCK_SYNCED) {
            t->free_hbm.push(id);
            released++;
        } else {
            if (r.slot[b] < 0) {
                if (t->free_slot.empty()) return false;
                r.slot[b] = t->free_slot.top();
                t->free_slot.pop();
            }
            t->oi.push_back(id);
            t->os.push_back(r.slot[b]);
            t->held.push_back(id);
        }
        r.hbm[b] = -1;
        r.state[b] = KV_BLOCK_HOST;
    }
    r.resident = false;
    r.n_full = 0;
    t->with_full.remove(q);
    return true;
}

// A request comes back: every block gets the lowest free HBM id and joins the in
// list; its slots stay its own.  False: the cache has no block left.
static bool enter_hbm(kv_table *t, int32_t q)
{
    save_request(t, q);
    TableReq &r = t->req[(size_t)q];
    for (size_t b = 0; b < r.hbm.size(); b++) {
        if (t->free_hbm.empty()) return false;
        const int32_t id = t->free_hbm.top();
        t->free_hbm.pop();
        r.hbm[b] = id;
        r.state[b] = KV_BLOCK_SYNCED;
        t->ii.push_back(id);
        t->is.push_back(r.slot[b]);
    }
    r.resident = true;
    return true;
}

// A rotation is a transaction on the table: the requests leave and enter as if
// the transfer had already been accepted, and whatever goes wrong on the way
// (no slot left, no block left, the engine refusing the transfer) ends in
// end_undo(false), which puts every request, both free sets and the counters
// back.  So there is no counting of room beforehand: running out is found by
// running out.
static int rotate_impl(kv_table *t, const int32_t *pre, int32_t n_pre, const int32_t *res, int32_t n_res,
                       int32_t eager_budget, int32_t *n_eager)
{
    if (!t || list_bad(pre, n_pre) || list_bad(res, n_res) || eager_budget < 0) return KV_EINVAL;
    if (!names_ok(t, pre, n_pre, res, n_res)) return KV_EINVAL;
    begin_undo(t);
    t->oi.clear(); t->os.clear(); t->ii.clear(); t->is.clear(); t->held.clear();
    int64_t released = 0;
    bool fits = true;
    for (int32_t i = 0; fits && i < n_pre; i++) fits = leave_hbm(t, pre[i], released);
    for (int32_t i = 0; fits && i < n_res; i++) fits = enter_hbm(t, res[i]);
    if (!fits) {
        end_undo(t, false);
        return KV_ENOSPC;
    }
    for (int32_t id : t->held) t->free_hbm.push(id);
    const size_t n_preempt_copies = t->oi.size();
    t->cnt.copied_preempt += (int64_t)n_preempt_copies;
    t->cnt.dropped_synced += released;
    t->cnt.swapped_in += (int64_t)t->ii.size();
    // the eager step of the requests that are resident now, riding in the same transfer
    std::vector<std::pair<int32_t, size_t>> picked;
    std::vector<int32_t> fresh;
    if (eager_budget > 0) {
        pick_eager(t, eager_budget, picked, fresh);
        mark_synced(t, picked, n_preempt_copies, true);
        t->cnt.copied_eager += (int64_t)picked.size();
    }
    // The lists are conflict-free by construction, so a refusal here is a shape the
    // path cannot serve or a HIP error; nothing was enqueued.
    const int rc = kv_rotate(t->e, t->oi.data(), t->os.data(), (int32_t)t->oi.size(), t->ii.data(), t->is.data(),
                             (int32_t)t->ii.size());
    end_undo(t, rc == KV_OK);
    if (rc == KV_OK) {
        for (int32_t i = 0; i < n_res; i++) t->req[(size_t)res[i]].named_at = (int64_t)t->e->idle_epoch;
        for (const auto &pk : picked) t->req[(size_t)pk.first].named_at = (int64_t)t->e->idle_epoch;
    }
    if (n_eager) *n_eager = rc == KV_OK ? (int32_t)picked.size() : 0;
    return rc;
}

int kv_table_rotate(kv_table *t, const int32_t *pre, int32_t n_pre, const int32_t *res, int32_t n_res)
{
    return rotate_impl(t, pre, n_pre, res, n_res, 0, nullptr);
}

int kv_table_rotate_eager(kv_table *t, const int32_t *pre, int32_t n_pre, const int32_t *res, int32_t n_res,
                          int32_t eager_budget, int32_t *n_eager)
{
    if (n_eager) *n_eager = 0;
    return rotate_impl(t, pre, n_pre, res, n_res, eager_budget, n_eager);
}

int kv_table_finish(kv_table *t, int32_t rq)
{
    if (!t || rq < 0 || rq >= t->max_req || !t->req[(size_t)rq].used) return KV_EINVAL;
    // Its HBM blocks go to new owners, who write them at once: a transfer that
    // still reads or writes them (an eager copy, its resumption) has to be done
    // first.  That can only be one enqueued since the engine was last seen idle.
    // (Host slots need no wait: only the engine's own, ordered transfers touch them.)
    TableReq &r = t->req[(size_t)rq];
    if (r.resident && r.named_at == (int64_t)t->e->idle_epoch) {
        const int rc = dkv::drain(t->e);
        if (rc != KV_OK) return rc;
    } else if (t->e->sticky != KV_OK) {
        return t->e->sticky;
    }
    for (size_t b = 0; b < r.hbm.size(); b++) {
        if (r.hbm[b] >= 0) t->free_hbm.push(r.hbm[b]);
        if (r.slot[b] >= 0) t->free_slot.push(r.slot[b]);
    }
    t->with_full.remove(rq);
    r = TableReq{};
    return KV_OK;
}

int kv_table_blocks(kv_table *t, int32_t rq, int32_t *ids, int32_t *slots, int32_t *states, int32_t cap,
                    int32_t *n, int32_t *info)
{
    if (!t || rq < 0 || rq >= t->max_req || !t->req[(size_t)rq].used || !n) return KV_EINVAL;
    const TableReq &r = t->req[(size_t)rq];
    if ((ids || slots || states) && (int64_t)r.hbm.size() > cap) return KV_EINVAL;
    for (size_t b = 0; b < r.hbm.size(); b++) {
        if (ids) ids[b] = r.hbm[b];
        if (slots) slots[b] = r.slot[b];
        if (states) states[b] = r.state[b];
    }
    *n = (int32_t)r.hbm.size();
    if (info) {
        info[0] = r.len;
        info[1] = r.resident ? 1 : 0;
    }
    return KV_OK;
}

int kv_table_get_counts(kv_table *t, kv_table_counts *out)
{
    if (!t || !out) return KV_EINVAL;
    *out = t->cnt;
    out->free_hbm_blocks = (int64_t)t->free_hbm.size();
    out->free_host_slots = (int64_t)t->free_slot.size();
    return KV_OK;
}

}  // extern "C"
