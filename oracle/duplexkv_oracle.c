/*
 * CPU oracle for paged-KV block rotation.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the plain definition the HIP path is checked against.  It is
 * used by the tests, by the smoke check and by the benchmark's CPU-baseline
 * leg, and by nothing else: the product path never calls it and shares no
 * source, header, table or helper with it.
 *
 * What is computed (paper Section 4.3.1 for the cache structure, Section 4.3.2
 * for the two directions): a KV cache holds, for each of N_L layers, a K plane
 * and a V plane, each an array of fixed-size blocks of P tokens.  The bytes of
 * one block inside one plane of one layer are the largest contiguous unit,
 * the "segment".  Swap-out copies every segment of the named HBM blocks to the
 * named host slots; swap-in copies every segment of the named host slots to
 * the named HBM blocks.  A rotation does both.  The method changes when and
 * how the bytes move, never which bytes, so the oracle is a memcpy per segment
 * in list order, with no blocking, fusion or reordering.
 *
 * HBM layouts : 0 = layer-first [layer][K|V][block][token][kv_head][dim]
 *               1 = block-first [block][layer][K|V][token][kv_head][dim], the
 *                   cache arrangement Section 4.3.2 proposes ("Block-first
 *                   layout and batched KV transfers": all layers of a block
 *                   contiguous, stride between blocks N_L x S_seg)
 * Host layouts: 0 = block-first [slot][layer][K|V][token][kv_head][dim]
 *                   (all layers of a block contiguous, the arrangement of
 *                   Section 4.3.2 "Block-first layout")
 *               1 = layer-first [layer][K|V][slot][token][kv_head][dim]
 *
 * Every function here is pinned by tests that do not go through this file's
 * own arithmetic: a six-loop element-wise brute force, a tagged-fill closed
 * form, array-indexing in NumPy, the round-trip / untouched / rejection
 * invariants and the worked sizes printed in Section 4.3.1.
 */
#include <pthread.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Result codes.  The values are part of the interface contract. */
enum {
    OKV_OK = 0,
    OKV_EINVAL = -1,   /* NULL list with n > 0, n < 0, bad shape            */
    OKV_ERANGE = -2,   /* an id outside [0, blocks) or [0, slots)            */
    OKV_EDUP = -3,     /* the same id twice inside one list                 */
    OKV_EOVERLAP = -4  /* a block or slot named for both directions         */
};

typedef struct {
    int32_t n_layers;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t block_size;   /* tokens per block, P */
    int32_t elem_bytes;   /* 2 for 16-bit KV */
    int32_t n_hbm_blocks;
    int32_t n_host_slots;
    int32_t host_layout;  /* 0 block-first, 1 layer-first */
    int32_t hbm_layout;   /* 0 layer-first, 1 block-first */
} okv_shape;

static int shape_ok(const okv_shape *s)
{
    return s && s->n_layers > 0 && s->n_kv_heads > 0 && s->head_dim > 0 &&
           s->block_size > 0 && s->elem_bytes > 0 && s->n_hbm_blocks > 0 &&
           s->n_host_slots > 0 && (s->host_layout == 0 || s->host_layout == 1) &&
           (s->hbm_layout == 0 || s->hbm_layout == 1);
}

/* Segment: P tokens x per-token bytes of one plane (Section 4.3.1, S_seg = P x C
 * with C split here into its K half and its V half). */
uint64_t okv_seg_bytes(const okv_shape *s)
{
    return (uint64_t)s->block_size * (uint64_t)s->n_kv_heads *
           (uint64_t)s->head_dim * (uint64_t)s->elem_bytes;
}

/* All layers, K and V, of one block: what one block costs on the link. */
uint64_t okv_block_bytes(const okv_shape *s)
{
    return 2u * (uint64_t)s->n_layers * okv_seg_bytes(s);
}

uint64_t okv_cache_bytes(const okv_shape *s)
{
    return okv_block_bytes(s) * (uint64_t)s->n_hbm_blocks;
}

uint64_t okv_pool_bytes(const okv_shape *s)
{
    return okv_block_bytes(s) * (uint64_t)s->n_host_slots;
}

/* Byte offset of segment (layer l, plane kv, block b) in the HBM image. */
uint64_t okv_hbm_offset(const okv_shape *s, int32_t l, int32_t kv, int32_t b)
{
    uint64_t plane = (uint64_t)l * 2u + (uint64_t)kv;
    uint64_t n_planes = 2u * (uint64_t)s->n_layers;
    if (s->hbm_layout == 1)
        return ((uint64_t)b * n_planes + plane) * okv_seg_bytes(s);
    return (plane * (uint64_t)s->n_hbm_blocks + (uint64_t)b) * okv_seg_bytes(s);
}

/* Byte offset of segment (layer l, plane kv, slot sl) in the host pool. */
uint64_t okv_pool_offset(const okv_shape *s, int32_t l, int32_t kv, int32_t sl)
{
    uint64_t plane = (uint64_t)l * 2u + (uint64_t)kv;
    uint64_t n_planes = 2u * (uint64_t)s->n_layers;
    if (s->host_layout == 0)
        return ((uint64_t)sl * n_planes + plane) * okv_seg_bytes(s);
    return (plane * (uint64_t)s->n_host_slots + (uint64_t)sl) * okv_seg_bytes(s);
}

static int list_bad(const int32_t *p, int32_t n) { return n < 0 || (n > 0 && !p); }

static int any_out_of_range(const int32_t *p, int32_t n, int32_t limit)
{
    for (int32_t i = 0; i < n; i++)
        if (p[i] < 0 || p[i] >= limit)
            return 1;
    return 0;
}

static int any_duplicate(const int32_t *p, int32_t n)
{
    for (int32_t i = 0; i < n; i++)
        for (int32_t j = i + 1; j < n; j++)
            if (p[i] == p[j])
                return 1;
    return 0;
}

static int any_common(const int32_t *a, int32_t na, const int32_t *b, int32_t nb)
{
    for (int32_t i = 0; i < na; i++)
        for (int32_t j = 0; j < nb; j++)
            if (a[i] == b[j])
                return 1;
    return 0;
}

/*
 * All-or-nothing admission of a rotation.  The swap-in destinations must not
 * coincide with the swap-out sources, which is the data race of Section 4.3.2
 * ("The challenge lies in swap-in/out dependencies"); the same holds on the
 * host side for slots.  Checks run in a fixed order so that an input that is
 * wrong in several ways always gets the same code:
 *   arguments, then ranges of all four lists, then duplicates inside each
 *   list, then overlap between the directions.
 */
int okv_validate(const okv_shape *s,
                 const int32_t *out_ids, const int32_t *out_slots, int32_t n_out,
                 const int32_t *in_ids, const int32_t *in_slots, int32_t n_in)
{
    if (!shape_ok(s))
        return OKV_EINVAL;
    if (list_bad(out_ids, n_out) || list_bad(out_slots, n_out) ||
        list_bad(in_ids, n_in) || list_bad(in_slots, n_in))
        return OKV_EINVAL;
    if (any_out_of_range(out_ids, n_out, s->n_hbm_blocks) ||
        any_out_of_range(in_ids, n_in, s->n_hbm_blocks) ||
        any_out_of_range(out_slots, n_out, s->n_host_slots) ||
        any_out_of_range(in_slots, n_in, s->n_host_slots))
        return OKV_ERANGE;
    if (any_duplicate(out_ids, n_out) || any_duplicate(out_slots, n_out) ||
        any_duplicate(in_ids, n_in) || any_duplicate(in_slots, n_in))
        return OKV_EDUP;
    if (any_common(out_ids, n_out, in_ids, n_in) ||
        any_common(out_slots, n_out, in_slots, n_in))
        return OKV_EOVERLAP;
    return OKV_OK;
}

/* One block HBM -> host: every layer, K then V, one segment at a time. */
static void block_out(const okv_shape *s, const uint8_t *hbm, uint8_t *pool,
                      int32_t id, int32_t slot)
{
    uint64_t seg = okv_seg_bytes(s);
    for (int32_t l = 0; l < s->n_layers; l++)
        for (int32_t kv = 0; kv < 2; kv++)
            memcpy(pool + okv_pool_offset(s, l, kv, slot),
                   hbm + okv_hbm_offset(s, l, kv, id), seg);
}

/* One block host -> HBM. */
static void block_in(const okv_shape *s, uint8_t *hbm, const uint8_t *pool,
                     int32_t id, int32_t slot)
{
    uint64_t seg = okv_seg_bytes(s);
    for (int32_t l = 0; l < s->n_layers; l++)
        for (int32_t kv = 0; kv < 2; kv++)
            memcpy(hbm + okv_hbm_offset(s, l, kv, id),
                   pool + okv_pool_offset(s, l, kv, slot), seg);
}

/*
 * Rotation: blocks out_ids[i] go to slots out_slots[i]; slots in_slots[j] come
 * back into blocks in_ids[j].  Source bytes are left as they are (copy, not
 * move).  On any admission error nothing is touched.  Because admission makes
 * the four id sets conflict-free, the order of the copies cannot change the
 * result: exactly one result is correct.
 */
int okv_rotate(const okv_shape *s, uint8_t *hbm, uint8_t *pool,
               const int32_t *out_ids, const int32_t *out_slots, int32_t n_out,
               const int32_t *in_ids, const int32_t *in_slots, int32_t n_in)
{
    int rc = okv_validate(s, out_ids, out_slots, n_out, in_ids, in_slots, n_in);
    if (rc != OKV_OK)
        return rc;
    if ((n_out > 0 || n_in > 0) && (!hbm || !pool))
        return OKV_EINVAL;
    for (int32_t i = 0; i < n_out; i++)
        block_out(s, hbm, pool, out_ids[i], out_slots[i]);
    for (int32_t j = 0; j < n_in; j++)
        block_in(s, hbm, pool, in_ids[j], in_slots[j]);
    return OKV_OK;
}

int okv_swap_out(const okv_shape *s, uint8_t *hbm, uint8_t *pool,
                 const int32_t *ids, const int32_t *slots, int32_t n)
{
    return okv_rotate(s, hbm, pool, ids, slots, n, NULL, NULL, 0);
}

int okv_swap_in(const okv_shape *s, uint8_t *hbm, uint8_t *pool,
                const int32_t *slots, const int32_t *ids, int32_t n)
{
    return okv_rotate(s, hbm, pool, NULL, NULL, 0, ids, slots, n);
}

/*
 * Synthetic decode reader (stands in for the model execution that runs while
 * blocks rotate, Section 4.3.2 "Cross-iteration pipeline"): what a pass over
 * the KV of the running requests reads.  The result is the sum, modulo 2^64,
 * of every little-endian 32-bit word of every segment (all layers, K and V)
 * of the named blocks; a block named twice counts twice.  Segment size must
 * be a multiple of 4 bytes.
 */
int okv_read_checksum(const okv_shape *s, const uint8_t *hbm, const int32_t *ids, int32_t n,
                      uint64_t *sum_out)
{
    if (!shape_ok(s) || list_bad(ids, n) || !sum_out || (n > 0 && !hbm))
        return OKV_EINVAL;
    if (okv_seg_bytes(s) % 4u != 0)
        return OKV_EINVAL;
    if (any_out_of_range(ids, n, s->n_hbm_blocks))
        return OKV_ERANGE;
    uint64_t sum = 0;
    uint64_t words = okv_seg_bytes(s) / 4u;
    for (int32_t l = 0; l < s->n_layers; l++)
        for (int32_t kv = 0; kv < 2; kv++)
            for (int32_t i = 0; i < n; i++) {
                const uint8_t *p = hbm + okv_hbm_offset(s, l, kv, ids[i]);
                for (uint64_t w = 0; w < words; w++) {
                    uint32_t v = (uint32_t)p[4 * w] | ((uint32_t)p[4 * w + 1] << 8) |
                                 ((uint32_t)p[4 * w + 2] << 16) | ((uint32_t)p[4 * w + 3] << 24);
                    sum += v;
                }
            }
    *sum_out = sum;
    return OKV_OK;
}

/*
 * The same rotation with the two block lists dealt out over host threads in
 * contiguous shares (thread t takes blocks [t*n/T, (t+1)*n/T) of each list).
 * Only the CPU-baseline timing uses this; the copies are the same calls.
 */
typedef struct {
    const okv_shape *s;
    uint8_t *hbm, *pool;
    const int32_t *out_ids, *out_slots, *in_ids, *in_slots;
    int32_t o0, o1, i0, i1;
} okv_share;

static void *share_main(void *arg)
{
    okv_share *w = (okv_share *)arg;
    for (int32_t i = w->o0; i < w->o1; i++)
        block_out(w->s, w->hbm, w->pool, w->out_ids[i], w->out_slots[i]);
    for (int32_t j = w->i0; j < w->i1; j++)
        block_in(w->s, w->hbm, w->pool, w->in_ids[j], w->in_slots[j]);
    return NULL;
}

int okv_rotate_threads(const okv_shape *s, uint8_t *hbm, uint8_t *pool,
                       const int32_t *out_ids, const int32_t *out_slots, int32_t n_out,
                       const int32_t *in_ids, const int32_t *in_slots, int32_t n_in,
                       int32_t n_threads)
{
    int rc = okv_validate(s, out_ids, out_slots, n_out, in_ids, in_slots, n_in);
    if (rc != OKV_OK)
        return rc;
    if (n_threads < 1 || ((n_out > 0 || n_in > 0) && (!hbm || !pool)))
        return OKV_EINVAL;
    pthread_t *tid = (pthread_t *)calloc((size_t)n_threads, sizeof(pthread_t));
    okv_share *sh = (okv_share *)calloc((size_t)n_threads, sizeof(okv_share));
    if (!tid || !sh) {
        free(tid);
        free(sh);
        return OKV_EINVAL;
    }
    for (int32_t t = 0; t < n_threads; t++) {
        okv_share w = { s, hbm, pool, out_ids, out_slots, in_ids, in_slots,
                        (int32_t)((int64_t)n_out * t / n_threads),
                        (int32_t)((int64_t)n_out * (t + 1) / n_threads),
                        (int32_t)((int64_t)n_in * t / n_threads),
                        (int32_t)((int64_t)n_in * (t + 1) / n_threads) };
        sh[t] = w;
        pthread_create(&tid[t], NULL, share_main, &sh[t]);
    }
    for (int32_t t = 0; t < n_threads; t++)
        pthread_join(tid[t], NULL);
    free(tid);
    free(sh);
    return OKV_OK;
}

/* ------------------------------------------------------------------------
 * Block table with eager block rotation (paper Section 4.3.2, "Eager block
 * rotation for data race free overlapping"), as a plain state machine.
 *
 * A request's KV grows token by token; a block that is still being filled is
 * DIRTY, a filled block is FULL until its copy to DRAM has been issued and
 * SYNCED afterwards (valid copies in HBM and in DRAM), and the blocks of a
 * preempted request are HOST (DRAM only).  The eager step copies FULL blocks
 * out in the background; at preemption only blocks without a valid DRAM copy
 * (the dirty tail, and any FULL block the eager step has not reached) are
 * copied, the HBM blocks of SYNCED ones are released at once without moving
 * a byte; a resumed request is copied back whole and keeps its DRAM copies,
 * so it is SYNCED again.  Blocks released by SYNCED drops may be reused by
 * the swap-ins of the same rotation; blocks that the same rotation copies out
 * may not (that is the race the section describes).
 *
 * Readings where the paper is silent: allocation takes the lowest-numbered
 * free HBM block / host slot; the eager step visits requests by ascending id
 * and blocks by ascending index; a request keeps its host slots until it
 * finishes; appending to a partly filled block makes it DIRTY again.
 * Everything is linear scans over small arrays: slow and easy to check.
 * ------------------------------------------------------------------------ */
enum { OKV_ENOSPC = -8 };
enum { OKVT_NONE = 0, OKVT_DIRTY = 1, OKVT_FULL = 2, OKVT_SYNCED = 3, OKVT_HOST = 4 };

typedef struct {
    int32_t used;      /* request exists */
    int32_t resident;  /* 1 running (in HBM), 0 rotary (in DRAM) */
    int32_t len;       /* tokens */
    int32_t n;         /* blocks */
    int32_t *hbm, *slot, *state;
} okvt_req;

typedef struct okvt {
    okv_shape s;
    int32_t max_req;
    okvt_req *req;
    int32_t *hbm_owner;  /* -1 free, else request id */
    int32_t *slot_owner;
    int64_t copied_eager, copied_preempt, dropped_synced, swapped_in;
} okvt;

okvt *okvt_create(const okv_shape *s, int32_t max_requests)
{
    if (!shape_ok(s) || max_requests <= 0)
        return NULL;
    okvt *t = (okvt *)calloc(1, sizeof(okvt));
    t->s = *s;
    t->max_req = max_requests;
    t->req = (okvt_req *)calloc((size_t)max_requests, sizeof(okvt_req));
    t->hbm_owner = (int32_t *)malloc(sizeof(int32_t) * (size_t)s->n_hbm_blocks);
    t->slot_owner = (int32_t *)malloc(sizeof(int32_t) * (size_t)s->n_host_slots);
    for (int32_t i = 0; i < s->n_hbm_blocks; i++) t->hbm_owner[i] = -1;
    for (int32_t i = 0; i < s->n_host_slots; i++) t->slot_owner[i] = -1;
    return t;
}

void okvt_destroy(okvt *t)
{
    if (!t) return;
    for (int32_t r = 0; r < t->max_req; r++) {
        free(t->req[r].hbm);
        free(t->req[r].slot);
        free(t->req[r].state);
    }
    free(t->req);
    free(t->hbm_owner);
    free(t->slot_owner);
    free(t);
}

static int32_t count_free(const int32_t *owner, int32_t n)
{
    int32_t c = 0;
    for (int32_t i = 0; i < n; i++) c += owner[i] < 0;
    return c;
}

static int32_t lowest_free(const int32_t *owner, int32_t n)
{
    for (int32_t i = 0; i < n; i++)
        if (owner[i] < 0) return i;
    return -1;
}

static int32_t blocks_for(const okvt *t, int32_t tokens)
{
    return (tokens + t->s.block_size - 1) / t->s.block_size;
}

/* Grow request `req` by n_tokens (creating it if it does not exist).  Reports
 * the HBM ids of blocks newly allocated for it.  All-or-nothing. */
int okvt_append(okvt *t, int32_t req, int32_t n_tokens, int32_t *new_ids, int32_t cap, int32_t *n_new)
{
    if (!t || req < 0 || req >= t->max_req || n_tokens < 0) return OKV_EINVAL;
    okvt_req *r = &t->req[req];
    if (r->used && !r->resident) return OKV_EINVAL; /* a rotary request cannot generate */
    int32_t old_n = r->used ? r->n : 0, old_len = r->used ? r->len : 0;
    int32_t need = blocks_for(t, old_len + n_tokens) - old_n;
    if (need > count_free(t->hbm_owner, t->s.n_hbm_blocks)) return OKV_ENOSPC;
    if (new_ids && need > cap) return OKV_EINVAL;
    if (!r->used) {
        r->used = 1;
        r->resident = 1;
        r->len = 0;
        r->n = 0;
        if (!r->hbm) {
            r->hbm = (int32_t *)malloc(sizeof(int32_t) * (size_t)t->s.n_hbm_blocks);
            r->slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)t->s.n_hbm_blocks);
            r->state = (int32_t *)malloc(sizeof(int32_t) * (size_t)t->s.n_hbm_blocks);
        }
    }
    /* tokens that land in the current tail block make it dirty again */
    if (n_tokens > 0 && old_len % t->s.block_size != 0) r->state[old_n - 1] = OKVT_DIRTY;
    for (int32_t k = 0; k < need; k++) {
        int32_t b = lowest_free(t->hbm_owner, t->s.n_hbm_blocks);
        t->hbm_owner[b] = req;
        r->hbm[r->n] = b;
        r->slot[r->n] = -1;
        r->state[r->n] = OKVT_DIRTY;
        if (new_ids) new_ids[k] = b;
        r->n++;
    }
    r->len = old_len + n_tokens;
    /* every block that is now completely filled and was being filled is FULL */
    for (int32_t i = 0; i < r->n; i++) {
        int32_t filled = (i + 1) * t->s.block_size <= r->len;
        if (filled && r->state[i] == OKVT_DIRTY) r->state[i] = OKVT_FULL;
    }
    if (n_new) *n_new = need;
    return OKV_OK;
}

/* Background step: copy up to `budget` FULL blocks of running requests to DRAM. */
int okvt_eager(okvt *t, uint8_t *hbm, uint8_t *pool, int32_t budget, int32_t *n_done)
{
    if (!t || budget < 0) return OKV_EINVAL;
    int32_t done = 0;
    for (int32_t q = 0; q < t->max_req && done < budget; q++) {
        okvt_req *r = &t->req[q];
        if (!r->used || !r->resident) continue;
        for (int32_t i = 0; i < r->n && done < budget; i++) {
            if (r->state[i] != OKVT_FULL) continue;
            if (r->slot[i] < 0) {
                int32_t sl = lowest_free(t->slot_owner, t->s.n_host_slots);
                if (sl < 0) goto out; /* pool exhausted: sync what fits */
                t->slot_owner[sl] = q;
                r->slot[i] = sl;
            }
            block_out(&t->s, hbm, pool, r->hbm[i], r->slot[i]);
            r->state[i] = OKVT_SYNCED;
            done++;
        }
    }
out:
    t->copied_eager += done;
    if (n_done) *n_done = done;
    return OKV_OK;
}

static int in_list(const int32_t *p, int32_t n, int32_t v)
{
    for (int32_t i = 0; i < n; i++)
        if (p[i] == v) return 1;
    return 0;
}

/* One rotation: `pre` requests leave HBM, `res` requests come back. */
int okvt_rotate(okvt *t, uint8_t *hbm, uint8_t *pool, const int32_t *pre, int32_t n_pre,
                const int32_t *res, int32_t n_res)
{
    if (!t || list_bad(pre, n_pre) || list_bad(res, n_res)) return OKV_EINVAL;
    for (int32_t i = 0; i < n_pre; i++) {
        if (pre[i] < 0 || pre[i] >= t->max_req) return OKV_EINVAL;
        okvt_req *r = &t->req[pre[i]];
        if (!r->used || !r->resident || in_list(pre, i, pre[i])) return OKV_EINVAL;
    }
    for (int32_t i = 0; i < n_res; i++) {
        if (res[i] < 0 || res[i] >= t->max_req) return OKV_EINVAL;
        okvt_req *r = &t->req[res[i]];
        if (!r->used || r->resident || in_list(res, i, res[i])) return OKV_EINVAL;
    }
    /* room check before anything changes */
    int32_t need_slots = 0, drop = 0, need_hbm = 0;
    for (int32_t i = 0; i < n_pre; i++) {
        okvt_req *r = &t->req[pre[i]];
        for (int32_t b = 0; b < r->n; b++) {
            if (r->state[b] == OKVT_SYNCED) drop++;
            else if (r->slot[b] < 0) need_slots++;
        }
    }
    for (int32_t i = 0; i < n_res; i++) need_hbm += t->req[res[i]].n;
    if (need_slots > count_free(t->slot_owner, t->s.n_host_slots)) return OKV_ENOSPC;
    if (need_hbm > count_free(t->hbm_owner, t->s.n_hbm_blocks) + drop) return OKV_ENOSPC;

    /* 1. preempted requests: blocks without a valid DRAM copy are copied out;
     *    SYNCED blocks give their HBM block back at once */
    int32_t n_out = 0;
    int32_t *held = (int32_t *)malloc(sizeof(int32_t) * (size_t)t->s.n_hbm_blocks);
    for (int32_t i = 0; i < n_pre; i++) {
        okvt_req *r = &t->req[pre[i]];
        for (int32_t b = 0; b < r->n; b++) {
            if (r->state[b] == OKVT_SYNCED) {
                t->hbm_owner[r->hbm[b]] = -1;
                t->dropped_synced++;
            } else {
                if (r->slot[b] < 0) {
                    int32_t sl = lowest_free(t->slot_owner, t->s.n_host_slots);
                    t->slot_owner[sl] = pre[i];
                    r->slot[b] = sl;
                }
                block_out(&t->s, hbm, pool, r->hbm[b], r->slot[b]);
                held[n_out++] = r->hbm[b]; /* stays unavailable during this rotation */
                t->copied_preempt++;
            }
            r->hbm[b] = -1;
            r->state[b] = OKVT_HOST;
        }
        r->resident = 0;
    }
    /* 2. resumed requests: every block comes back into the lowest free HBM block */
    for (int32_t i = 0; i < n_res; i++) {
        okvt_req *r = &t->req[res[i]];
        for (int32_t b = 0; b < r->n; b++) {
            int32_t id = lowest_free(t->hbm_owner, t->s.n_hbm_blocks);
            t->hbm_owner[id] = res[i];
            r->hbm[b] = id;
            block_in(&t->s, hbm, pool, id, r->slot[b]);
            r->state[b] = OKVT_SYNCED;
            t->swapped_in++;
        }
        r->resident = 1;
    }
    /* 3. the copied-out blocks are free from now on */
    for (int32_t k = 0; k < n_out; k++) t->hbm_owner[held[k]] = -1;
    free(held);
    return OKV_OK;
}

/* A rotation with the eager step of the requests that stay riding along
 * (Section 4.3.2: eager copies are issued while other transfers run).  Defined
 * as what it must equal: the rotation, then the eager step. */
int okvt_rotate_eager(okvt *t, uint8_t *hbm, uint8_t *pool, const int32_t *pre, int32_t n_pre,
                      const int32_t *res, int32_t n_res, int32_t eager_budget, int32_t *n_eager)
{
    if (n_eager) *n_eager = 0;
    if (eager_budget < 0) return OKV_EINVAL;
    int rc = okvt_rotate(t, hbm, pool, pre, n_pre, res, n_res);
    if (rc != OKV_OK) return rc;
    return okvt_eager(t, hbm, pool, eager_budget, n_eager);
}

/* The request is done: its HBM blocks and host slots are free again. */
int okvt_finish(okvt *t, int32_t req)
{
    if (!t || req < 0 || req >= t->max_req || !t->req[req].used) return OKV_EINVAL;
    okvt_req *r = &t->req[req];
    for (int32_t b = 0; b < r->n; b++) {
        if (r->hbm[b] >= 0) t->hbm_owner[r->hbm[b]] = -1;
        if (r->slot[b] >= 0) t->slot_owner[r->slot[b]] = -1;
    }
    r->used = 0;
    r->n = 0;
    r->len = 0;
    return OKV_OK;
}

/* Mapping and state of a request's blocks; info = {len_tokens, resident}. */
int okvt_blocks(const okvt *t, int32_t req, int32_t *ids, int32_t *slots, int32_t *states, int32_t cap,
                int32_t *n, int32_t *info)
{
    if (!t || req < 0 || req >= t->max_req || !t->req[req].used || !n) return OKV_EINVAL;
    const okvt_req *r = &t->req[req];
    if (r->n > cap) return OKV_EINVAL;
    for (int32_t b = 0; b < r->n; b++) {
        if (ids) ids[b] = r->hbm[b];
        if (slots) slots[b] = r->slot[b];
        if (states) states[b] = r->state[b];
    }
    *n = r->n;
    if (info) {
        info[0] = r->len;
        info[1] = r->resident;
    }
    return OKV_OK;
}

/* counts = {free HBM blocks, free host slots, blocks copied by the eager step,
 * blocks copied at preemption, SYNCED blocks dropped without a copy, blocks swapped in} */
int okvt_counts(const okvt *t, int64_t *counts)
{
    if (!t || !counts) return OKV_EINVAL;
    counts[0] = count_free(t->hbm_owner, t->s.n_hbm_blocks);
    counts[1] = count_free(t->slot_owner, t->s.n_host_slots);
    counts[2] = t->copied_eager;
    counts[3] = t->copied_preempt;
    counts[4] = t->dropped_synced;
    counts[5] = t->swapped_in;
    return OKV_OK;
}

/* ------------------------------------------------------------------------
 * Scheduler that decides what rotates: Virtual Lag Time and Largest-VLT-First
 * (paper Section 4.2.1, the VLT equation, and Section 4.2.2, Algorithm 1).
 *
 * VLT of a request at time t_now:
 *   rotary : alpha * ReLU(t_now - t_last - beta_B * S_B)
 *   waiting:         ReLU(t_now - t_arr  - beta_F * S_F)
 *   running:        -(t_now - t_run)
 * Reading of the garbled sentence under the equation: the equation pairs S_B
 * with rotary requests, which wait for their next token, so S_B is the
 * time-between-tokens SLO, and S_F with waiting requests, so S_F is the
 * time-to-first-token SLO.
 *
 * LVF, in the algorithm's order: contention check (if the free HBM blocks hold
 * every waiting and rotary request, prioritise them all, first come first
 * served, and preempt nobody); sort all requests by VLT, largest first; walk
 * from the head and prioritise waiting / rotary requests with VLT >= 0 that
 * still fit into B_HBM + B_xfer blocks; B_swap = B_xfer - B_left; walk from
 * the tail and preempt running requests with VLT < 0 while B_swap > 0.
 * Readings: ties in VLT are broken by ascending request id; only waiting and
 * rotary requests can be prioritised (a running request whose VLT is exactly
 * 0 is already in HBM); first come first served orders by the request's
 * reference time (arrival, or last token), then id.
 * ------------------------------------------------------------------------ */
enum { OKV_RUNNING = 0, OKV_WAITING = 1, OKV_ROTARY = 2 };

typedef struct {
    double alpha, beta_b, beta_f; /* sensitivity weight and the two tolerance coefficients */
    double slo_tbt, slo_ttft;     /* S_B and S_F, seconds */
} okv_sched_params;

typedef struct {
    int32_t id;
    int32_t state;  /* OKV_RUNNING / WAITING / ROTARY */
    int32_t blocks; /* blk(r) */
    int32_t pad;
    double t_ref;   /* running: t_run; waiting: t_arr; rotary: t_last */
} okv_sched_req;

static double relu(double x) { return x > 0.0 ? x : 0.0; }

double okv_sched_vlt(const okv_sched_params *p, const okv_sched_req *r, double t_now)
{
    if (r->state == OKV_ROTARY) return p->alpha * relu(t_now - r->t_ref - p->beta_b * p->slo_tbt);
    if (r->state == OKV_WAITING) return relu(t_now - r->t_ref - p->beta_f * p->slo_ttft);
    return -(t_now - r->t_ref);
}

/* preempt[] / prioritize[] receive request ids in the order they were chosen
 * (room for n each).  *fcfs = 1 if the contention check short-circuited. */
int okv_sched_lvf(const okv_sched_params *p, const okv_sched_req *reqs, int32_t n, double t_now,
                  int32_t b_xfer, int32_t b_hbm, int32_t *preempt, int32_t *n_preempt,
                  int32_t *prioritize, int32_t *n_prioritize, int32_t *fcfs)
{
    if (!p || n < 0 || (n > 0 && !reqs) || b_xfer < 0 || b_hbm < 0 || !n_preempt || !n_prioritize ||
        (n > 0 && (!preempt || !prioritize)))
        return OKV_EINVAL;
    for (int32_t i = 0; i < n; i++)
        if (reqs[i].state < OKV_RUNNING || reqs[i].state > OKV_ROTARY || reqs[i].blocks < 0)
            return OKV_EINVAL;
    *n_preempt = 0;
    *n_prioritize = 0;
    if (fcfs) *fcfs = 0;
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    double *vlt = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    for (int32_t i = 0; i < n; i++) {
        order[i] = i;
        vlt[i] = okv_sched_vlt(p, &reqs[i], t_now);
    }
    /* step 1: contention check */
    int64_t need = 0;
    for (int32_t i = 0; i < n; i++)
        if (reqs[i].state != OKV_RUNNING) need += reqs[i].blocks;
    if ((int64_t)b_hbm >= need) {
        /* first come first served: insertion sort by (t_ref, id) */
        for (int32_t a = 1; a < n; a++)
            for (int32_t b = a; b > 0; b--) {
                const okv_sched_req *x = &reqs[order[b - 1]], *y = &reqs[order[b]];
                if (x->t_ref > y->t_ref || (x->t_ref == y->t_ref && x->id > y->id)) {
                    int32_t t = order[b]; order[b] = order[b - 1]; order[b - 1] = t;
                } else break;
            }
        for (int32_t i = 0; i < n; i++)
            if (reqs[order[i]].state != OKV_RUNNING) prioritize[(*n_prioritize)++] = reqs[order[i]].id;
        if (fcfs) *fcfs = 1;
        free(order);
        free(vlt);
        return OKV_OK;
    }
    /* step 2: sort by VLT, largest first (ties: smaller id first) */
    for (int32_t a = 1; a < n; a++)
        for (int32_t b = a; b > 0; b--) {
            int32_t x = order[b - 1], y = order[b];
            if (vlt[x] < vlt[y] || (vlt[x] == vlt[y] && reqs[x].id > reqs[y].id)) {
                order[b] = x; order[b - 1] = y;
            } else break;
        }
    /* step 3: prioritise from the head */
    int64_t left = (int64_t)b_hbm + b_xfer;
    for (int32_t i = 0; i < n; i++) {
        const okv_sched_req *r = &reqs[order[i]];
        if (r->state != OKV_RUNNING && vlt[order[i]] >= 0.0 && r->blocks <= left) {
            prioritize[(*n_prioritize)++] = r->id;
            left -= r->blocks;
        }
    }
    /* step 4: preempt from the tail */
    int64_t swap = (int64_t)b_xfer - left;
    for (int32_t i = n - 1; i >= 0; i--) {
        const okv_sched_req *r = &reqs[order[i]];
        if (r->state == OKV_RUNNING && vlt[order[i]] < 0.0 && swap > 0) {
            preempt[(*n_preempt)++] = r->id;
            swap -= r->blocks;
        }
    }
    free(order);
    free(vlt);
    return OKV_OK;
}
