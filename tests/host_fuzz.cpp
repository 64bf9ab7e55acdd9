// CPU-only differential fuzz of the library's host logic: the block table of
// eager block rotation (paper Section 4.3.2) and the VLT / LVF scheduler
// (Section 4.2, Algorithm 1) are driven with long random operation sequences
// side by side with the oracle's, and every return code, mapping, state,
// counter and byte is compared after every operation.  Meant to be built with
// -fsanitize=address,undefined, so memory errors in either side abort the run.
//
// The table's two engine calls are replaced here by a host stand-in that
// checks each transfer list for range, duplicates and overlap and then moves
// whole blocks between two byte arrays; no GPU and no HIP call is involved.
// The cache and the pool are block-first in this test, which makes a block one
// contiguous run of bytes on both sides.
#include <cinttypes>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "../paper_2601_20309_amd/csrc/kv_engine.hpp"

// ---- the oracle's interface (plain C, declared here as its source defines it)
extern "C" {
typedef struct {
    int32_t n_layers, n_kv_heads, head_dim, block_size, elem_bytes, n_hbm_blocks, n_host_slots, host_layout,
        hbm_layout;
} okv_shape;
typedef struct okvt okvt;
okvt *okvt_create(const okv_shape *s, int32_t max_requests);
void okvt_destroy(okvt *t);
int okvt_append(okvt *t, int32_t req, int32_t n_tokens, int32_t *new_ids, int32_t cap, int32_t *n_new);
int okvt_eager(okvt *t, uint8_t *hbm, uint8_t *pool, int32_t budget, int32_t *n_done);
int okvt_rotate(okvt *t, uint8_t *hbm, uint8_t *pool, const int32_t *pre, int32_t n_pre, const int32_t *res,
                int32_t n_res);
int okvt_rotate_eager(okvt *t, uint8_t *hbm, uint8_t *pool, const int32_t *pre, int32_t n_pre, const int32_t *res,
                      int32_t n_res, int32_t eager_budget, int32_t *n_eager);
int okvt_finish(okvt *t, int32_t req);
int okvt_blocks(const okvt *t, int32_t req, int32_t *ids, int32_t *slots, int32_t *states, int32_t cap, int32_t *n,
                int32_t *info);
int okvt_counts(const okvt *t, int64_t *counts);
uint64_t okv_block_bytes(const okv_shape *s);
typedef struct {
    double alpha, beta_b, beta_f, slo_tbt, slo_ttft;
} okv_sched_params;
typedef struct {
    int32_t id, state, blocks, pad;
    double t_ref;
} okv_sched_req;
double okv_sched_vlt(const okv_sched_params *p, const okv_sched_req *r, double t_now);
int okv_sched_lvf(const okv_sched_params *p, const okv_sched_req *reqs, int32_t n, double t_now, int32_t b_xfer,
                  int32_t b_hbm, int32_t *preempt, int32_t *n_preempt, int32_t *prioritize, int32_t *n_prioritize,
                  int32_t *fcfs);
}

#define CHECK(cond, ...)                                         \
    do {                                                         \
        if (!(cond)) {                                           \
            std::fprintf(stderr, "FAIL %s:%d: ", __FILE__, __LINE__); \
            std::fprintf(stderr, __VA_ARGS__);                   \
            std::fprintf(stderr, "\n");                          \
            std::exit(1);                                        \
        }                                                        \
    } while (0)

// ---- host stand-in for the engine's two calls the table makes
namespace {
uint64_t g_block_bytes = 0;
std::vector<uint8_t> g_hbm, g_pool;
int64_t g_transfers = 0;
// When not KV_OK: the next transfer call is refused with this code and moves nothing
// (an engine failure after the table has done its bookkeeping).
int g_fail_next = KV_OK;
int64_t g_refused = 0;

void check_list(const int32_t *a, int32_t n, int32_t limit, std::vector<int> &mark, int bit)
{
    for (int32_t i = 0; i < n; i++) {
        CHECK(a[i] >= 0 && a[i] < limit, "table issued id %d outside [0,%d)", a[i], limit);
        CHECK(!(mark[(size_t)a[i]] & bit), "table issued id %d twice in one list", a[i]);
        CHECK(!(mark[(size_t)a[i]] & ~bit), "table named id %d for both directions", a[i]);
        mark[(size_t)a[i]] |= bit;
    }
}
}  // namespace

extern "C" int kv_rotate(kv_engine *e, const int32_t *oi, const int32_t *os, int32_t no, const int32_t *ii,
                         const int32_t *is, int32_t ni)
{
    if (g_fail_next != KV_OK) {
        const int rc = g_fail_next;
        g_fail_next = KV_OK;
        g_refused++;
        return rc;
    }
    std::vector<int> mb((size_t)e->cfg.n_hbm_blocks, 0), ms((size_t)e->cfg.n_host_slots, 0);
    check_list(oi, no, e->cfg.n_hbm_blocks, mb, 1);
    check_list(ii, ni, e->cfg.n_hbm_blocks, mb, 2);
    check_list(os, no, e->cfg.n_host_slots, ms, 1);
    check_list(is, ni, e->cfg.n_host_slots, ms, 2);
    for (int32_t k = 0; k < no; k++)
        std::memcpy(&g_pool[(size_t)os[k] * g_block_bytes], &g_hbm[(size_t)oi[k] * g_block_bytes], g_block_bytes);
    for (int32_t k = 0; k < ni; k++)
        std::memcpy(&g_hbm[(size_t)ii[k] * g_block_bytes], &g_pool[(size_t)is[k] * g_block_bytes], g_block_bytes);
    g_transfers++;
    return KV_OK;
}

extern "C" int kv_swap_out(kv_engine *e, const int32_t *ids, const int32_t *slots, int32_t n)
{
    return kv_rotate(e, ids, slots, n, nullptr, nullptr, 0);
}

// the stand-in's transfers are done when the call returns
int dkv::drain(kv_engine *) { return KV_OK; }

// ---- table fuzz
namespace {

constexpr int32_t kCap = 256;  // blocks a request of the fuzz may reach

struct Pair {
    kv_table *lib = nullptr;
    okvt *ora = nullptr;
    okv_shape s{};
    int32_t max_req = 0;
    std::vector<uint8_t> o_hbm, o_pool;
    std::vector<int32_t> written;  // tokens of each request the "model" has written so far
};

// The model's part: tokens [from, to) of request q get their bytes, in both caches.
void write_tokens(Pair &p, int32_t q, int32_t from, int32_t to, std::mt19937_64 &rng)
{
    int32_t ids[kCap], n = 0;
    CHECK(kv_table_blocks(p.lib, q, ids, nullptr, nullptr, kCap, &n, nullptr) == KV_OK, "blocks");
    const uint64_t tok_bytes = g_block_bytes / (uint64_t)p.s.block_size;
    for (int32_t tkn = from; tkn < to; tkn++) {
        const int32_t b = ids[tkn / p.s.block_size];
        CHECK(b >= 0, "append left a token without an HBM block");
        const size_t off = (size_t)b * g_block_bytes + (size_t)(tkn % p.s.block_size) * tok_bytes;
        for (uint64_t k = 0; k < tok_bytes; k++) {
            const uint8_t v = (uint8_t)rng();
            g_hbm[off + k] = v;
            p.o_hbm[off + k] = v;
        }
    }
}

void compare(Pair &p, long step, const char *op)
{
    int32_t la[kCap], lb[kCap], lc[kCap], oa[kCap], ob[kCap], oc[kCap];
    for (int32_t q = 0; q < p.max_req; q++) {
        int32_t ln = -1, on = -1, li[2] = {-1, -1}, oi[2] = {-1, -1};
        const int rl = kv_table_blocks(p.lib, q, la, lb, lc, kCap, &ln, li);
        const int ro = okvt_blocks(p.ora, q, oa, ob, oc, kCap, &on, oi);
        CHECK(rl == ro, "step %ld (%s) req %d: blocks() returned %d, oracle %d", step, op, q, rl, ro);
        if (rl != KV_OK) continue;
        CHECK(ln == on && li[0] == oi[0] && li[1] == oi[1], "step %ld (%s) req %d: n %d/%d len %d/%d resident %d/%d",
              step, op, q, ln, on, li[0], oi[0], li[1], oi[1]);
        for (int32_t b = 0; b < ln; b++)
            CHECK(la[b] == oa[b] && lb[b] == ob[b] && lc[b] == oc[b],
                  "step %ld (%s) req %d block %d: id %d/%d slot %d/%d state %d/%d", step, op, q, b, la[b], oa[b],
                  lb[b], ob[b], lc[b], oc[b]);
    }
    kv_table_counts c{};
    int64_t oc6[6];
    CHECK(kv_table_get_counts(p.lib, &c) == KV_OK && okvt_counts(p.ora, oc6) == 0, "counts");
    CHECK(c.free_hbm_blocks == oc6[0] && c.free_host_slots == oc6[1] && c.copied_eager == oc6[2] &&
              c.copied_preempt == oc6[3] && c.dropped_synced == oc6[4] && c.swapped_in == oc6[5],
          "step %ld (%s): counters differ: free %" PRId64 "/%" PRId64 " slots %" PRId64 "/%" PRId64
          " eager %" PRId64 "/%" PRId64 " preempt %" PRId64 "/%" PRId64 " dropped %" PRId64 "/%" PRId64
          " in %" PRId64 "/%" PRId64,
          step, op, c.free_hbm_blocks, oc6[0], c.free_host_slots, oc6[1], c.copied_eager, oc6[2], c.copied_preempt,
          oc6[3], c.dropped_synced, oc6[4], c.swapped_in, oc6[5]);
    CHECK(g_hbm == p.o_hbm, "step %ld (%s): cache bytes differ", step, op);
    CHECK(g_pool == p.o_pool, "step %ld (%s): pool bytes differ", step, op);
}

// reach_id: the run must hand out a block id at least this high (so that the id
// sets of the library are exercised beyond their first words)
long fuzz_table(uint64_t seed, long steps, int32_t nb, int32_t ns, int32_t max_req, int32_t P, int32_t reach_id = 0)
{
    int32_t top_id = -1;
    std::mt19937_64 rng(seed);
    Pair p;
    p.s = okv_shape{1, 1, 4, P, 2, nb, ns, 0, 1};
    p.max_req = max_req;
    g_block_bytes = okv_block_bytes(&p.s);
    CHECK(g_block_bytes == (uint64_t)2 * P * 4 * 2, "block bytes");
    g_hbm.assign((size_t)nb * g_block_bytes, 0);
    g_pool.assign((size_t)ns * g_block_bytes, 0);
    for (auto &v : g_hbm) v = (uint8_t)rng();
    for (auto &v : g_pool) v = (uint8_t)rng();
    p.o_hbm = g_hbm;
    p.o_pool = g_pool;
    p.written.assign((size_t)max_req, 0);

    kv_engine eng{};
    eng.cfg.n_layers = 1, eng.cfg.n_kv_heads = 1, eng.cfg.head_dim = 4, eng.cfg.block_size = P;
    eng.cfg.elem_bytes = 2, eng.cfg.n_hbm_blocks = nb, eng.cfg.n_host_slots = ns;
    eng.cfg.path = KV_PATH_FUSED;
    CHECK(kv_table_create(&p.lib, &eng, max_req) == KV_OK, "create");
    p.ora = okvt_create(&p.s, max_req);
    CHECK(p.ora, "oracle create");

    long failed_ops = 0;
    // a table that starts out well filled: requests of 60 blocks until the ids wanted are in use
    for (int32_t q = 0; reach_id > 0 && top_id < reach_id; q++) {
        CHECK(q < max_req, "not enough requests to reach block id %d", reach_id);
        int32_t li[64], oi[64], ln = -7, on = -7;
        const int rl = kv_table_append(p.lib, q, 60 * P, li, 64, &ln);
        const int ro = okvt_append(p.ora, q, 60 * P, oi, 64, &on);
        CHECK(rl == KV_OK && ro == KV_OK && ln == 60 && on == 60, "filling: %d / %d, %d / %d blocks", rl, ro, ln, on);
        for (int32_t k = 0; k < ln; k++) {
            CHECK(li[k] == oi[k], "filling: new id differs");
            top_id = std::max(top_id, li[k]);
        }
        write_tokens(p, q, 0, 60 * P, rng);
        p.written[(size_t)q] = 60 * P;
        compare(p, -1, "fill");
    }
    for (long step = 0; step < steps; step++) {
        const unsigned pick = (unsigned)(rng() % 100);
        const char *op = "";
        if (pick < 45) {  // grow or create a request
            op = "append";
            const int32_t q = (int32_t)(rng() % (uint64_t)(max_req + 1)) - (rng() % 64 == 0);  // sometimes invalid
            int32_t n_tok = (int32_t)(rng() % (uint64_t)(3 * P + 1)) - (rng() % 97 == 0);
            if (q >= 0 && q < max_req && n_tok > 0 && p.written[(size_t)q] + n_tok > (kCap - 1) * P) n_tok = 0;
            int32_t li[64], oi[64], ln = -7, on = -7;
            const int rl = kv_table_append(p.lib, q, n_tok, li, 64, &ln);
            const int ro = okvt_append(p.ora, q, n_tok, oi, 64, &on);
            CHECK(rl == ro, "step %ld append(%d,%d): %d, oracle %d", step, q, n_tok, rl, ro);
            if (rl == KV_OK) {
                CHECK(ln == on, "step %ld append: %d new blocks, oracle %d", step, ln, on);
                for (int32_t k = 0; k < ln; k++) CHECK(li[k] == oi[k], "step %ld append: new id differs", step);
                for (int32_t k = 0; k < ln; k++) top_id = std::max(top_id, li[k]);
                write_tokens(p, q, p.written[(size_t)q], p.written[(size_t)q] + n_tok, rng);
                p.written[(size_t)q] += n_tok;
            } else
                failed_ops++;
        } else if (pick < 65) {
            op = "eager";
            const int32_t budget = (int32_t)(rng() % 9) - (rng() % 53 == 0);
            int32_t ln = -7, on = -7;
            const bool inject = rng() % 20 == 0;
            const int64_t refused = g_refused;
            if (inject) g_fail_next = KV_EHIP;
            const int rl = kv_table_eager(p.lib, budget, &ln);
            g_fail_next = KV_OK;
            if (g_refused != refused) {
                // the engine refused the copies: the table must be what it was (the oracle never hears of it)
                op = "eager, transfer refused";
                CHECK(rl == KV_EHIP, "step %ld eager with a refused transfer returned %d", step, rl);
                failed_ops++;
            } else {
                const int ro = okvt_eager(p.ora, p.o_hbm.data(), p.o_pool.data(), budget, &on);
                CHECK(rl == ro, "step %ld eager(%d): %d, oracle %d", step, budget, rl, ro);
                if (rl == KV_OK) CHECK(ln == on, "step %ld eager: %d copied, oracle %d", step, ln, on);
                else failed_ops++;
            }
        } else if (pick < 90) {
            op = "rotate";
            // random subsets, usually of the right kind, sometimes not
            std::vector<int32_t> pre, res;
            for (int32_t q = 0; q < max_req; q++) {
                int32_t n = 0, info[2] = {0, 0};
                const bool used = kv_table_blocks(p.lib, q, nullptr, nullptr, nullptr, 0, &n, info) == KV_OK;
                const bool wrong = rng() % 200 == 0;
                if ((used && info[1] == 1) != wrong && rng() % 4 == 0) pre.push_back(q);
                else if ((used && info[1] == 0) != wrong && rng() % 3 == 0) res.push_back(q);
            }
            if (rng() % 150 == 0 && !pre.empty()) res.push_back(pre[0]);  // named twice
            if (rng() % 150 == 0) pre.push_back(max_req + 3);             // out of range
            int rl, ro;
            if (rng() % 16 == 0) {
                // The engine refuses the transfer after the table has worked out the whole
                // rotation: every mapping, state, free list and counter must be as before.
                op = "rotate, transfer refused";
                const int64_t refused = g_refused;
                const int code = rng() % 2 ? KV_EHIP : KV_EUNSUP;
                g_fail_next = code;
                int32_t ln = -7;
                if (rng() % 2)
                    rl = kv_table_rotate(p.lib, pre.data(), (int32_t)pre.size(), res.data(), (int32_t)res.size());
                else
                    rl = kv_table_rotate_eager(p.lib, pre.data(), (int32_t)pre.size(), res.data(),
                                               (int32_t)res.size(), (int32_t)(rng() % 7), &ln);
                g_fail_next = KV_OK;
                if (g_refused != refused) {
                    CHECK(rl == code, "step %ld: refused transfer came back as %d", step, rl);
                    CHECK(ln == -7 || ln == 0, "step %ld: %d eager copies reported for a refused transfer", step, ln);
                } else {
                    CHECK(rl != KV_OK, "step %ld: a rotation succeeded without asking the engine", step);
                }
                ro = rl;  // the oracle is not told: its table is the "before" the library must still equal
            } else if (rng() % 2) {
                rl = kv_table_rotate(p.lib, pre.data(), (int32_t)pre.size(), res.data(), (int32_t)res.size());
                ro = okvt_rotate(p.ora, p.o_hbm.data(), p.o_pool.data(), pre.data(), (int32_t)pre.size(), res.data(),
                                 (int32_t)res.size());
            } else {  // the eager step in the same transfer
                op = "rotate_eager";
                const int32_t budget = (int32_t)(rng() % 7) - (rng() % 41 == 0);
                int32_t ln = -7, on = -7;
                const int64_t before = g_transfers;
                rl = kv_table_rotate_eager(p.lib, pre.data(), (int32_t)pre.size(), res.data(), (int32_t)res.size(),
                                           budget, &ln);
                ro = okvt_rotate_eager(p.ora, p.o_hbm.data(), p.o_pool.data(), pre.data(), (int32_t)pre.size(),
                                       res.data(), (int32_t)res.size(), budget, &on);
                CHECK(ln == on, "step %ld rotate_eager: %d eager copies, oracle %d", step, ln, on);
                CHECK(g_transfers - before == (rl == KV_OK ? 1 : 0), "rotate_eager issued %ld transfers",
                      (long)(g_transfers - before));
            }
            CHECK(rl == ro, "step %ld %s(%zu,%zu): %d, oracle %d", step, op, pre.size(), res.size(), rl, ro);
            if (rl != KV_OK) failed_ops++;
        } else {
            op = "finish";
            const int32_t q = (int32_t)(rng() % (uint64_t)(max_req + 1)) - (rng() % 64 == 0);
            const int rl = kv_table_finish(p.lib, q);
            const int ro = okvt_finish(p.ora, q);
            CHECK(rl == ro, "step %ld finish(%d): %d, oracle %d", step, q, rl, ro);
            if (rl == KV_OK) p.written[(size_t)q] = 0;
            else failed_ops++;
        }
        compare(p, step, op);
    }
    kv_table_counts c{};
    kv_table_get_counts(p.lib, &c);
    std::printf("table seed %" PRIu64 ": %ld ops (%ld refused), %" PRId64 " transfers, eager %" PRId64
                " preempt %" PRId64 " dropped %" PRId64 " in %" PRId64 "\n",
                seed, steps, failed_ops, g_transfers, c.copied_eager, c.copied_preempt, c.dropped_synced,
                c.swapped_in);
    CHECK(c.copied_eager > 0 && c.copied_preempt > 0 && c.dropped_synced > 0 && c.swapped_in > 0,
          "the fuzz never reached one of the four kinds of block movement");
    CHECK(g_refused > 0, "the fuzz never refused a transfer");
    CHECK(top_id >= reach_id, "the fuzz only reached block id %d of the %d wanted", top_id, reach_id);
    CHECK(kv_table_destroy(p.lib) == KV_OK, "destroy");
    okvt_destroy(p.ora);
    return failed_ops;
}

// ---- scheduler fuzz: same inputs to both, same selections out
void fuzz_sched(uint64_t seed, long rounds)
{
    std::mt19937_64 rng(seed);
    std::uniform_real_distribution<double> u01(0.0, 1.0);
    long n_fcfs = 0, n_pre = 0, n_pri = 0, n_bad = 0;
    for (long it = 0; it < rounds; it++) {
        const int32_t n = (int32_t)(rng() % 40);
        kv_sched_params lp{};
        lp.alpha = (rng() % 5 == 0) ? 0.0 : 4.0 * u01(rng);
        lp.beta_b = 2.0 * u01(rng), lp.beta_f = 2.0 * u01(rng);
        lp.slo_tbt = 0.2 * u01(rng), lp.slo_ttft = 3.0 * u01(rng);
        okv_sched_params op{lp.alpha, lp.beta_b, lp.beta_f, lp.slo_tbt, lp.slo_ttft};
        const double t_now = 10.0 + 5.0 * u01(rng);
        std::vector<kv_sched_req> lr((size_t)n);
        std::vector<okv_sched_req> orq((size_t)n);
        const bool coarse = rng() % 3 == 0;  // coarse times make ties, which the id must break
        for (int32_t i = 0; i < n; i++) {
            lr[(size_t)i].id = 100 + i;
            lr[(size_t)i].state = (int32_t)(rng() % 3);
            lr[(size_t)i].blocks = (int32_t)(rng() % 12);
            lr[(size_t)i].pad = 0;
            double t = t_now - 6.0 * u01(rng);
            if (coarse) t = (double)(long)(t * 2.0) / 2.0;
            lr[(size_t)i].t_ref = t;
            if (rng() % 400 == 0) lr[(size_t)i].state = 7;  // invalid
            orq[(size_t)i] = okv_sched_req{lr[(size_t)i].id, lr[(size_t)i].state, lr[(size_t)i].blocks, 0, t};
            if (lr[(size_t)i].state <= 2) {
                const double a = kv_sched_vlt(&lp, &lr[(size_t)i], t_now), b = okv_sched_vlt(&op, &orq[(size_t)i], t_now);
                CHECK(a == b, "sched seed %" PRIu64 " round %ld: VLT %a, oracle %a", seed, it, a, b);
            }
        }
        const int32_t b_xfer = (int32_t)(rng() % 40), b_hbm = (int32_t)(rng() % 80);
        std::vector<int32_t> lpre((size_t)n + 1, -5), lpri((size_t)n + 1, -5), opre((size_t)n + 1, -5),
            opri((size_t)n + 1, -5);
        int32_t lnp = -1, lnq = -1, lf = -1, onp = -1, onq = -1, of = -1;
        const int rl = kv_sched_lvf(&lp, lr.data(), n, t_now, b_xfer, b_hbm, lpre.data(), &lnp, lpri.data(), &lnq, &lf);
        const int ro = okv_sched_lvf(&op, orq.data(), n, t_now, b_xfer, b_hbm, opre.data(), &onp, opri.data(), &onq,
                                     &of);
        CHECK(rl == ro, "sched seed %" PRIu64 " round %ld: rc %d, oracle %d", seed, it, rl, ro);
        if (rl != KV_OK) {
            n_bad++;
            continue;
        }
        CHECK(lnp == onp && lnq == onq && lf == of, "sched seed %" PRIu64 " round %ld: counts %d/%d %d/%d fcfs %d/%d",
              seed, it, lnp, onp, lnq, onq, lf, of);
        for (int32_t i = 0; i < lnp; i++) CHECK(lpre[(size_t)i] == opre[(size_t)i], "preempt[%d] differs", i);
        for (int32_t i = 0; i < lnq; i++) CHECK(lpri[(size_t)i] == opri[(size_t)i], "prioritize[%d] differs", i);
        CHECK(lpre[(size_t)n] == -5 && lpri[(size_t)n] == -5, "scheduler wrote past n entries");
        n_fcfs += lf, n_pre += lnp, n_pri += lnq;
    }
    std::printf("sched seed %" PRIu64 ": %ld rounds (%ld refused), fcfs %ld, preempted %ld, prioritized %ld\n", seed,
                rounds, n_bad, n_fcfs, n_pre, n_pri);
    CHECK(n_fcfs > 0 && n_fcfs < rounds && n_pre > 0 && n_pri > 0, "scheduler fuzz missed a branch");
}

}  // namespace

int main(int argc, char **argv)
{
    const long steps = argc > 1 ? std::atol(argv[1]) : 20000;
    const long rounds = argc > 2 ? std::atol(argv[2]) : 20000;
    // plenty of room; tight HBM; tight host pool; one-token blocks
    fuzz_table(1, steps, 24, 40, 10, 4);
    fuzz_table(2, steps, 9, 40, 10, 4);
    fuzz_table(3, steps, 24, 11, 10, 4);
    fuzz_table(4, steps, 16, 24, 6, 1);
    // id sets of several words; of several summary words (ids beyond 4096)
    fuzz_table(7, steps, 300, 500, 150, 2, 200);
    fuzz_table(8, steps, 6000, 9000, 700, 1, 4200);
    fuzz_sched(5, rounds);
    fuzz_sched(6, rounds);
    std::printf("host fuzz ok\n");
    return 0;
}
