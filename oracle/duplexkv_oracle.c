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
 * HBM layout  : [layer][K|V][block][token][kv_head][dim]
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
} okv_shape;

static int shape_ok(const okv_shape *s)
{
    return s && s->n_layers > 0 && s->n_kv_heads > 0 && s->head_dim > 0 &&
           s->block_size > 0 && s->elem_bytes > 0 && s->n_hbm_blocks > 0 &&
           s->n_host_slots > 0 && (s->host_layout == 0 || s->host_layout == 1);
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
