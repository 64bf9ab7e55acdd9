/*
 * duplexkv.h - C ABI of the MI355X KV-cache rotation engine.
 *
 * The engine moves paged KV blocks between a cache in HBM and a pinned block
 * pool in host memory, out and in at the same time, which is the job of the
 * rotation engine of the SuperInfer paper (Section 4.3.2, "Efficient KV Cache
 * Rotation Engine"; cache structure from Section 4.3.1).  The link here is
 * PCIe Gen5 x16, not NVLink-C2C, so the transfer design is this library's own.
 *
 * Vocabulary (Section 4.3.1): the cache has N_L layers, each with a K plane and
 * a V plane; a plane is an array of blocks of P tokens; the bytes of one block
 * in one plane are one "segment", the largest contiguous unit in HBM:
 *   seg   = block_size * n_kv_heads * head_dim * elem_bytes
 *   block = 2 * n_layers * seg          (what one block costs on the link)
 * HBM layout : KV_HBM_LAYER_FIRST [layer][K|V][block][token][kv_head][dim] (default;
 *              K = 0, V = 1), or KV_HBM_BLOCK_FIRST [block][layer][K|V][token]...,
 *              the cache arrangement Section 4.3.2 proposes (a block is one
 *              contiguous region, stride between blocks N_L x S_seg per plane pair).
 * Host pool  : KV_HOST_BLOCK_FIRST [slot][layer][K|V][token][kv_head][dim]
 *              (all layers of a block contiguous: the "block-first layout" of
 *              Section 4.3.2) or KV_HOST_LAYER_FIRST [layer][K|V][slot][...].
 *
 * Conventions for every call
 *  - returns 0 (KV_OK) or a negative KV_E* code; kv_strerror() names it.
 *  - id arrays are host memory owned by the caller, read before the call
 *    returns (the caller may free them at once); int32, unpadded.
 *  - the transfer calls only enqueue work; kv_wait() completes it.
 *  - admission is all-or-nothing: on any error no byte of cache or pool has
 *    been modified and nothing was enqueued.
 *  - an engine is used from one host thread at a time.
 */
#ifndef DUPLEXKV_H
#define DUPLEXKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- result codes ---- */
#define KV_OK         0
#define KV_EINVAL   (-1)  /* NULL argument, n < 0, NULL list with n > 0, bad config */
#define KV_ERANGE   (-2)  /* block id outside [0, n_hbm_blocks) or slot outside [0, n_host_slots) */
#define KV_EDUP     (-3)  /* the same id twice within one list */
#define KV_EOVERLAP (-4)  /* a block id, or a slot, named for both directions of one call */
#define KV_ENOMEM   (-5)  /* a device or pinned-host allocation failed */
#define KV_EHIP     (-6)  /* HIP runtime failure (no device, launch or copy error); sticky */
#define KV_EUNSUP   (-7)  /* the chosen path cannot serve this shape or request */
#define KV_ENOSPC   (-8)  /* block table: not enough free HBM blocks or host slots */
#define KV_EBUSY    (-9)  /* a block or slot is still used the other way round by an un-waited call on the other stream */
#define KV_E2BIG    (-10) /* kv_rotate_static: more blocks than its scratch array holds */

/* ---- host pool layouts ---- */
#define KV_HOST_BLOCK_FIRST 0
#define KV_HOST_LAYER_FIRST 1

/* ---- cache layouts ---- */
#define KV_HBM_LAYER_FIRST 0
#define KV_HBM_BLOCK_FIRST 1

/* ---- transfer paths ---- */
#define KV_PATH_AUTO        0  /* engine picks: FUSED for a rotation, ZEROCOPY for one direction */
#define KV_PATH_SDMA_STAGED 1  /* pack kernel -> staging in HBM -> hipMemcpyAsync (DMA engines), and the mirror: ~10 % slower
                                  than the kernel paths, and takes a third as much from an HBM-bound kernel running beside it */
#define KV_PATH_ZEROCOPY    2  /* one kernel per direction, each on its own stream, reading / writing host memory directly */
#define KV_PATH_NAIVE       3  /* one hipMemcpyAsync per segment: the baseline of Section 4.3.1, for the benchmark ladder */
#define KV_PATH_FUSED       4  /* one kernel moves both directions, interleaved per lane: 1:1, or, when the in list is the
                                  longer one, with the out tiles spread evenly over the in tiles */
#define KV_PATH_DMA_BLOCKS  5  /* one hipMemcpyAsync per block (runs of consecutive ids and slots merge): the
                                  "merged segments" design of Section 4.3.2; needs KV_HBM_BLOCK_FIRST and KV_HOST_BLOCK_FIRST */

typedef struct kv_engine kv_engine; /* opaque, owned by the library */

typedef struct {
    int32_t n_layers;      /* N_L */
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t block_size;    /* P, tokens per block */
    int32_t elem_bytes;    /* 2 for bf16 / fp16 KV */
    int32_t n_hbm_blocks;  /* blocks per plane in the HBM cache */
    int32_t n_host_slots;  /* block slots in the host pool */
    int32_t host_layout;   /* KV_HOST_* */
    int32_t path;          /* KV_PATH_* */
    int32_t chunk_layers;  /* layers per chunk: DMA-staged path, 0 = engine picks; kernel paths, 0 = one launch, c > 0 =
                              c layers per launch with a completion mark each (kv_stream_wait_layer) */
    int32_t max_copy_wgs;  /* workgroups (of wg_lanes lanes; of 256 if wg_lanes is 0) a copy kernel may occupy; 0 = engine picks */
    int32_t vecs_per_lane; /* 16-byte vectors each lane keeps in flight per direction in the link kernels: 0 = engine picks, else 1, 2, 4 or 8 */
    int32_t wg_lanes;      /* lanes per workgroup of the link kernels (workgroups only pack waves; a wave is the unit of work):
                              0 = engine picks (with max_copy_wgs also 0: 112 one-wave workgroups), else a multiple of 64 up to 1024 */
    int32_t hbm_layout;    /* KV_HBM_* */
    uint64_t staging_bytes;/* SDMA_STAGED: bytes of HBM staging per direction = largest chunk; 0 = engine picks (256 MiB) */
} kv_config;

typedef struct {
    uint64_t bytes_out;    /* bytes moved HBM -> host since the previous kv_wait */
    uint64_t bytes_in;     /* bytes moved host -> HBM since the previous kv_wait */
    double ms_out;         /* device time of the out work, first start to last end (HIP events on its stream) */
    double ms_in;          /* same for the in work */
    double ms_e2e;         /* host wall time, entry of the first transfer call to return of kv_wait */
    int32_t path_used;     /* KV_PATH_* of the last call */
    int32_t n_launches;    /* kernels + copies enqueued since the previous kv_wait */
} kv_stats;

/* ---- sizes (pure host arithmetic; Section 4.3.1, S_seg = P x C) ---- */
uint64_t kv_seg_bytes(const kv_config *cfg);    /* one segment */
uint64_t kv_block_bytes(const kv_config *cfg);  /* 2 * n_layers segments */
uint64_t kv_cache_bytes(const kv_config *cfg);  /* whole HBM cache */
uint64_t kv_pool_bytes(const kv_config *cfg);   /* whole host pool */

/*
 * Admission check of a rotation, host only (no GPU is touched).  The swap-in
 * destinations may not coincide with the swap-out sources: that is the data
 * race of Section 4.3.2; the same rule is applied to host slots.  Order of the
 * checks: arguments (KV_EINVAL), ranges of all four lists (KV_ERANGE),
 * duplicates within each list (KV_EDUP), overlap between directions
 * (KV_EOVERLAP).  A list may be NULL iff its n is 0.
 */
int kv_validate(const kv_config *cfg,
                const int32_t *out_block_ids, const int32_t *out_host_slots, int32_t n_out,
                const int32_t *in_block_ids, const int32_t *in_host_slots, int32_t n_in);

/*
 * Create an engine on the current HIP device.
 *  hbm_cache  : device pointer, kv_cache_bytes(cfg) bytes in the configured HBM layout;
 *               owned by the caller and must outlive the engine.
 *  host_pool  : NULL = the engine allocates (and owns) a pinned pool of
 *               kv_pool_bytes(cfg); otherwise a caller-owned pinned, device-mapped
 *               host pointer of that size (hipHostMalloc memory or a PyTorch
 *               pinned tensor).
 *  stream_out, stream_in : hipStream_t to enqueue on, or NULL = the engine
 *               creates (and owns) two non-blocking streams of default priority.
 * Fails with KV_EINVAL (bad config / pointers too small), KV_ENOMEM, KV_EHIP.
 */
int kv_create(kv_engine **engine, const kv_config *cfg, void *hbm_cache, void *host_pool,
              void *stream_out, void *stream_in);

/* Waits for outstanding work, then frees everything the engine owns.  KV_EBUSY,
 * with nothing done, while a block table created on the engine still exists. */
int kv_destroy(kv_engine *engine);

/*
 * Swap-out (Section 4.3.2, HBM -> DRAM): block block_ids[i] of every layer and
 * both planes is copied to host slot host_slots[i].  Source bytes stay as they
 * are.  Asynchronous: ordered on stream_out.
 */
int kv_swap_out(kv_engine *engine, const int32_t *block_ids, const int32_t *host_slots, int32_t n);

/*
 * Swap-in (Section 4.3.2, DRAM -> HBM): host slot host_slots[i] is copied into
 * block block_ids[i], which the caller promises is free.  Asynchronous: ordered
 * on stream_in.
 */
int kv_swap_in(kv_engine *engine, const int32_t *host_slots, const int32_t *block_ids, int32_t n);

/*
 * Duplex rotation (Section 4.3.2, simultaneous D2H/H2D): both of the above in
 * one call, running at the same time.  Admission as in kv_validate().  After
 * the call returns, later work on stream_out is ordered after the out copies
 * and later work on stream_in after the in copies.  Two calls that have not
 * been separated by kv_wait() run in enqueue order per stream, and the two
 * streams run side by side.  A call that would read a block or slot which an
 * un-waited call on the other stream writes, or write one which such a call
 * reads, is refused with KV_EBUSY and enqueues nothing (kv_swap_out / kv_swap_in
 * likewise).  A rotation that runs as one launch for both directions (the
 * default path with both lists non-empty) is ordered after everything enqueued
 * before it and before everything enqueued after it, so such rotations can
 * follow one another, over the same blocks too, without a wait.
 * The id lists of calls in flight live in a ring of 8 descriptor sets: the
 * ninth call without a kv_wait() in between blocks the host until the oldest of
 * them has finished on the GPU (so do kv_swap_out / kv_swap_in).
 */
int kv_rotate(kv_engine *engine,
              const int32_t *out_block_ids, const int32_t *out_host_slots, int32_t n_out,
              const int32_t *in_block_ids, const int32_t *in_host_slots, int32_t n_in);

/*
 * kv_rotate() for callers that cannot allocate: code under HIP graph capture,
 * tight serving loops that must not reach hipMalloc, harnesses that forbid it.
 * No engine: the caller passes the configuration (shape, layouts and, if
 * wanted, the launch-shape fields; path must be KV_PATH_AUTO or KV_PATH_FUSED),
 * the cache (device pointer, kv_cache_bytes), the pool (pinned, device-mapped
 * host pointer, kv_pool_bytes) and the hipStream_t to enqueue on (NULL = the
 * default stream), all on the current device.  The call allocates nothing, on
 * the device or through any library: the move kernel's step counters and the
 * device copy of the four id lists live in a fixed array of device memory that
 * belongs to the library (64 KiB + 256 bytes per GPU, held until the process
 * ends), which bounds a call to n_out + n_in <= KV_STATIC_MAX_BLOCKS (KV_E2BIG
 * beyond that; nothing enqueued).  Admission and result are kv_rotate's: one
 * launch carries both directions (or the one that is not empty).  Asynchronous:
 * the id lists are read before the call returns; completion is the stream's
 * (hipStreamSynchronize, or an event of the caller's).  Every call on a GPU
 * shares that GPU's array, so calls on one GPU must be ordered one after the
 * other (the same stream, or streams the caller orders): two calls that overlap
 * in time race on the id lists.  Host threads that call at the same time take
 * turns on a lock (the enqueue order is then theirs to define).  No
 * KV_EBUSY tracking: ordering against other work on the same blocks is the
 * stream's order.  The call may be recorded into a HIP graph (stream capture)
 * once one call on that device has been made outside any capture (the first
 * call looks up the array's device address); the id lists are then part of the
 * recording, and a replay moves what the blocks and slots hold at that moment.
 */
#define KV_STATIC_MAX_BLOCKS 8192
int kv_rotate_static(const kv_config *cfg, void *hbm_cache, void *host_pool, void *stream,
                     const int32_t *out_block_ids, const int32_t *out_host_slots, int32_t n_out,
                     const int32_t *in_block_ids, const int32_t *in_host_slots, int32_t n_in);

/* Blocks until everything enqueued so far is done; the host pool is then
 * coherent for CPU reads.  Closes the interval kv_last_stats() reports. */
int kv_wait(kv_engine *engine);

/* The same question without blocking, for a loop that polls between other work
 * (the engine loop of Section 4.3.2 prepares iteration t+1 while transfers run):
 * KV_OK when everything enqueued so far is done (kv_wait would return at once;
 * blocks swapped in may be read, host slots written may be read by the CPU),
 * KV_EBUSY while something still runs.  The stats interval stays open until
 * kv_wait; once KV_OK has been returned, lists that overlap the finished work
 * are accepted again (no KV_EBUSY for a race that can no longer happen). */
int kv_query(kv_engine *engine);

/*
 * Layer by layer (north_star: "per-layer chunking so that the transfers
 * overlap"; the paper overlaps the rotation for iteration t+1 with the execution
 * of iteration t, Section 4.3.2).  With cfg.chunk_layers = c > 0 the kernel paths
 * (KV_PATH_FUSED, KV_PATH_ZEROCOPY, and KV_PATH_AUTO, which picks one of them)
 * move a call's blocks c layers at a time, lowest layers first, one launch per
 * chunk, and mark the end of every chunk.  A consumer can then start on layer l
 * while the layers behind it still move:
 *   kv_stream_wait_layer: work enqueued on `stream` (a hipStream_t of the
 *     caller's, e.g. the model's compute stream) after this call starts only
 *     once layer `layer` of the most recent transfer call is in place: K and V
 *     of that layer of every block the call names, in both directions.
 *   kv_wait_layer: the same for the host; it blocks until then.  The stats
 *     interval stays open (only kv_wait closes it).
 * KV_PATH_SDMA_STAGED marks its chunks the same way when a chunk is chunk_layers
 * layers of the whole list (the staging buffer holds that much).  After a call
 * that did not run layer by layer (chunk_layers 0, a list cut to fit the staging
 * buffer, the per-copy DMA paths) both wait for the whole call.  KV_EINVAL for a layer outside
 * [0, n_layers).  The chunks cost a launch each (a few microseconds between
 * launches and a ramp per launch): meant for large rotations, where a chunk is
 * tens of MiB or more.  A mark is never seen early; it can be seen late: the
 * process's streams share a few hardware queues, and a consumer stream that
 * shares one with the engine's stream runs behind the launches already queued
 * there.
 */
int kv_stream_wait_layer(kv_engine *engine, void *stream, int32_t layer);
int kv_wait_layer(kv_engine *engine, int32_t layer);

/* Host address and size of the pool (for filling / checking it from the CPU). */
int kv_host_pool(kv_engine *engine, void **ptr, uint64_t *bytes);

/* Figures for the calls between the last two kv_wait()s. */
int kv_last_stats(kv_engine *engine, kv_stats *out);

/*
 * Host-link peak with plain pinned hipMemcpyAsync of `bytes` per direction on
 * the current device: the denominator the rotation is judged against, measured
 * the way Appendix B measures its link (copy-engine memcpy, one direction and
 * both at once, median of `reps`).  Outputs in GB/s (1e9 bytes per second);
 * the *_duplex figures are per direction while both run, best of several
 * stream pairings (streams share a few hardware queues).
 */
int kv_probe_link(uint64_t bytes, int32_t reps, double *d2h, double *h2d,
                  double *d2h_duplex, double *h2d_duplex);

/*
 * Synthetic decode reader: the stand-in for the model execution that runs
 * while blocks rotate (Section 4.3.2, "Cross-iteration pipeline to overlap
 * execution with rotation").  Streams every segment of the named HBM blocks,
 * layer by layer, `passes` times (1..256), on a stream of the engine's own so
 * that it overlaps kv_rotate, and reduces what it read to the sum modulo 2^64
 * of all little-endian 32-bit words (a block named twice counts twice; n may
 * be up to twice n_hbm_blocks).  Read only.  Needs segments that are multiples of 16 bytes (KV_EUNSUP otherwise).
 * max_wgs caps its persistent workgroups (0 = engine picks).  One reader at a time:
 * kv_reader_wait() must come before the next kv_reader_start().
 * The reader is not ordered against transfers and takes no part in the
 * KV_EBUSY bookkeeping: a block that a swap-in overwrites while a pass reads it
 * enters the sum with old, new or mixed bytes (nothing else is affected, the
 * reader writes nothing to the cache).  A caller who wants a defined sum names
 * blocks no un-waited swap-in targets, as a decode step only attends over
 * requests that are resident.
 */
int kv_reader_start(kv_engine *engine, const int32_t *block_ids, int32_t n, int32_t passes, int32_t max_wgs);

/*
 * Waits for the reader.  checksum: the sum over all passes.  ms_per_pass: NULL
 * or an array of `passes` doubles, device time of each pass (HIP events).
 */
int kv_reader_wait(kv_engine *engine, uint64_t *checksum, double *ms_per_pass);

/* ------------------------------------------------------------------------
 * Block table with eager block rotation (Section 4.3.2, "Eager block rotation
 * for data race free overlapping").  The table owns the allocation of the
 * engine's HBM blocks and host slots and tracks, per block of every request,
 * state and residency:
 *   KV_BLOCK_DIRTY   still being filled; HBM only
 *   KV_BLOCK_FULL    filled, copy to DRAM not yet issued; HBM only
 *   KV_BLOCK_SYNCED  valid copies in HBM and in DRAM
 *   KV_BLOCK_HOST    DRAM only (request preempted)
 * Allocation always takes the lowest-numbered free block / slot.  A request
 * keeps its host slots until kv_table_finish().  All calls only enqueue
 * transfers on the engine's streams; kv_wait() on the engine completes them.
 * Transfers the table issues are ordered so that a block or slot is never
 * overwritten while an earlier transfer still reads it.  While a table exists
 * the engine's kv_swap_out / kv_swap_in / kv_rotate must not be called.
 * Request ids are 0 .. max_requests-1.
 * ------------------------------------------------------------------------ */
#define KV_BLOCK_DIRTY  1
#define KV_BLOCK_FULL   2
#define KV_BLOCK_SYNCED 3
#define KV_BLOCK_HOST   4

typedef struct kv_table kv_table; /* opaque, owned by the library */

typedef struct {
    int64_t free_hbm_blocks, free_host_slots;
    int64_t copied_eager;    /* blocks copied out by kv_table_eager */
    int64_t copied_preempt;  /* blocks copied out at preemption (no valid DRAM copy yet) */
    int64_t dropped_synced;  /* HBM blocks released at preemption without moving a byte */
    int64_t swapped_in;      /* blocks copied back at resumption */
} kv_table_counts;

int kv_table_create(kv_table **table, kv_engine *engine, int32_t max_requests);
int kv_table_destroy(kv_table *table);

/*
 * Request `req` grows by n_tokens (it is created if new, and must be resident).
 * HBM blocks are allocated as needed; new_block_ids (NULL, or room for `cap`
 * ids) receives them and *n_new their count.  The caller then writes the new
 * tokens' KV into the request's blocks.  Tokens that land in a partly filled
 * block make it DIRTY; a block that fills up becomes FULL.  KV_ENOSPC, with
 * nothing changed, if the cache has too few free blocks.
 * A block handed out here may be one that a preemption released while its copy
 * to DRAM is still in flight: the caller's writes (which the engine's streams
 * know nothing of) have to come after the transfers enqueued so far, i.e. after
 * kv_wait(), kv_query() == KV_OK, or on a stream that waited through
 * kv_stream_wait_layer(stream, n_layers - 1).  In the cross-iteration pipeline
 * of Section 4.3.2 that is the case anyway: iteration t+1 starts when its
 * rotation has landed.
 */
int kv_table_append(kv_table *table, int32_t req, int32_t n_tokens, int32_t *new_block_ids, int32_t cap,
                    int32_t *n_new);

/*
 * Eager rotation step: enqueue the copy to DRAM of up to `budget` FULL blocks
 * of resident requests (ascending request id, then block index); they become
 * SYNCED.  Stops early when the pool is exhausted.  *n_done = blocks issued.
 */
int kv_table_eager(kv_table *table, int32_t budget, int32_t *n_done);

/*
 * One rotation: the `preempt` requests leave HBM, the `resume` requests come
 * back, as one duplex transfer.  Of a preempted request only blocks without a
 * valid DRAM copy are copied (the dirty tail, FULL blocks the eager step has
 * not reached); its SYNCED blocks are released at once and may be reused by
 * this very call's swap-ins, while the blocks being copied out may not (the
 * data race of Section 4.3.2).  A resumed request is copied back whole and is
 * SYNCED.  KV_EINVAL for unknown / duplicated / wrongly placed requests,
 * KV_ENOSPC if slots or blocks do not suffice; nothing changes on error.
 */
int kv_table_rotate(kv_table *table, const int32_t *preempt, int32_t n_preempt, const int32_t *resume,
                    int32_t n_resume);

/*
 * kv_table_rotate() and, in the same duplex transfer, kv_table_eager(eager_budget)
 * over the requests that are resident once the rotation is done: the result
 * (mappings, states, counters, bytes) is that of the two calls one after the
 * other.  Why one transfer: with eager block rotation a rotation copies little
 * out and much in, and on the host link swap-out bytes up to about 0.8 times
 * the swap-in bytes travel in the time the swap-in needs anyway, so eager
 * copies issued here cost no link time.  *n_eager (may be NULL) = eager copies
 * issued.  Errors as kv_table_rotate, and KV_EINVAL for a negative budget;
 * nothing changes on error.
 */
int kv_table_rotate_eager(kv_table *table, const int32_t *preempt, int32_t n_preempt, const int32_t *resume,
                          int32_t n_resume, int32_t eager_budget, int32_t *n_eager);

/* The request is done: its HBM blocks and host slots are free again.  If a
 * transfer that names HBM blocks of this request (an eager copy, its
 * resumption) may still be in flight, the call first waits for the engine's
 * transfers, so it can block the host; finishing a request whose blocks no
 * transfer has named since the engine was last idle never waits.  It does not
 * close the interval kv_last_stats() reports. */
int kv_table_finish(kv_table *table, int32_t req);

/* Mapping of a request: per block HBM id (-1 if none), host slot (-1 if
 * none), state; arrays may be NULL, else hold `cap` entries.  info[0] =
 * tokens, info[1] = 1 if resident. */
int kv_table_blocks(kv_table *table, int32_t req, int32_t *block_ids, int32_t *host_slots, int32_t *states,
                    int32_t cap, int32_t *n, int32_t *info);

int kv_table_get_counts(kv_table *table, kv_table_counts *out);

/* ------------------------------------------------------------------------
 * What rotates: Virtual Lag Time and Largest-VLT-First scheduling (paper
 * Section 4.2.1, the VLT equation, and Section 4.2.2, Algorithm 1).  Host only.
 *   VLT = alpha * ReLU(t_now - t_last - beta_b * slo_tbt)   rotary
 *         ReLU(t_now - t_arr - beta_f * slo_ttft)           waiting
 *         -(t_now - t_run)                                  running
 * kv_sched_lvf: if the b_hbm free blocks hold every waiting and rotary
 * request, all of them are prioritised first come first served (*fcfs = 1)
 * and nobody is preempted.  Otherwise requests are sorted by VLT, largest
 * first (ties: smaller id); waiting / rotary requests with VLT >= 0 are
 * prioritised from the head while they fit into b_hbm + b_xfer blocks; then
 * running requests with VLT < 0 are preempted from the tail while
 * b_swap = b_xfer - blocks left is positive.  preempt[] and prioritize[]
 * (room for n ids each) receive request ids in the order chosen; they are
 * what kv_table_rotate() takes.
 * ------------------------------------------------------------------------ */
#define KV_REQ_RUNNING 0
#define KV_REQ_WAITING 1
#define KV_REQ_ROTARY  2

typedef struct {
    double alpha;    /* sensitivity weight of rotary (between-token) lag, >= 0 */
    double beta_b;   /* tolerance coefficient on slo_tbt */
    double beta_f;   /* tolerance coefficient on slo_ttft */
    double slo_tbt;  /* S_B: time-between-tokens SLO, seconds */
    double slo_ttft; /* S_F: time-to-first-token SLO, seconds */
} kv_sched_params;

typedef struct {
    int32_t id;
    int32_t state;   /* KV_REQ_* */
    int32_t blocks;  /* blk(r): KV blocks the request holds or needs */
    int32_t pad;
    double t_ref;    /* running: t_run; waiting: t_arr; rotary: t_last (seconds) */
} kv_sched_req;

double kv_sched_vlt(const kv_sched_params *params, const kv_sched_req *req, double t_now);

int kv_sched_lvf(const kv_sched_params *params, const kv_sched_req *reqs, int32_t n, double t_now,
                 int32_t b_xfer, int32_t b_hbm, int32_t *preempt, int32_t *n_preempt, int32_t *prioritize,
                 int32_t *n_prioritize, int32_t *fcfs);

const char *kv_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* DUPLEXKV_H */
