// Internal definitions shared by the engine (duplexkv.hip) and the block table
// (kv_table.cpp): the engine object itself.  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <utility>
#include <vector>

#include "../../include/duplexkv.h"

namespace dkv {

// Admission marks (host only).
// mark[] holds (epoch << 2) | bits, bits: 1 = named by the out list, 2 = by the in list.
struct Marks {
    std::vector<uint32_t> blk, slot;
    uint32_t epoch = 0;
    void reset(size_t nb, size_t ns) { blk.assign(nb, 0); slot.assign(ns, 0); epoch = 0; }
    void next()
    {
        if (++epoch >= (1u << 30)) {
            std::fill(blk.begin(), blk.end(), 0u);
            std::fill(slot.begin(), slot.end(), 0u);
            epoch = 1;
        }
    }
};

// What un-waited calls still use, for refusing a call that would race with one
// of them.  Work on one stream runs in order; the two streams run side by side
// until something joins them (kv_wait, or a launch that carries both
// directions).  A stamp equal to `epoch` means: used since the last join.
struct Hazards {
    std::vector<uint32_t> blk_read, blk_written, slot_read, slot_written;  // by stream_out / stream_in work
    uint32_t epoch = 1;
    void reset(size_t nb, size_t ns)
    {
        blk_read.assign(nb, 0); blk_written.assign(nb, 0);
        slot_read.assign(ns, 0); slot_written.assign(ns, 0);
        epoch = 1;
    }
    void join()
    {
        if (++epoch == 0xFFFFFFFFu) reset(blk_read.size(), slot_read.size());
    }
    // out part: reads blocks, writes slots, on stream_out; in part: reads slots,
    // writes blocks, on stream_in.  Ids are in range (admission came first).
    bool races(const int32_t *oi, const int32_t *os, int32_t no, const int32_t *ii, const int32_t *is,
               int32_t ni) const
    {
        for (int32_t k = 0; k < no; k++)
            if (blk_written[(size_t)oi[k]] == epoch || slot_read[(size_t)os[k]] == epoch) return true;
        for (int32_t k = 0; k < ni; k++)
            if (blk_read[(size_t)ii[k]] == epoch || slot_written[(size_t)is[k]] == epoch) return true;
        return false;
    }
    void stamp(const int32_t *oi, const int32_t *os, int32_t no, const int32_t *ii, const int32_t *is, int32_t ni)
    {
        for (int32_t k = 0; k < no; k++) { blk_read[(size_t)oi[k]] = epoch; slot_written[(size_t)os[k]] = epoch; }
        for (int32_t k = 0; k < ni; k++) { blk_written[(size_t)ii[k]] = epoch; slot_read[(size_t)is[k]] = epoch; }
    }
};

constexpr int kRing = 8;  // descriptor sets that may be in flight
// Tile counters of the link-bound kernels: one pair per stream (launches on a
// stream run one after the other), each pair in a 256-byte stretch of its own.
constexpr int kClaimStride = 64;

inline bool list_bad(const int32_t *p, int32_t n) { return n < 0 || (n > 0 && !p); }

}  // namespace dkv

struct kv_engine;
namespace dkv {
// Blocks until the transfers enqueued so far are done, without closing the
// interval kv_last_stats() reports (kv_wait does that).  No-op when nothing is
// pending.  Defined with the engine; the block table calls it before it hands
// blocks and slots of a finished request to new owners.
int drain(kv_engine *e);
}  // namespace dkv

struct kv_engine {
    kv_config cfg;
    int device = 0;
    uint64_t seg = 0, block_bytes = 0, cache_bytes = 0, pool_bytes = 0;
    uint32_t n_planes = 0;
    int vec = 1;  // bytes per lane access
    uint8_t *hbm = nullptr;
    uint8_t *pool = nullptr;
    bool own_pool = false;
    hipStream_t s_out = nullptr, s_in = nullptr;
    bool own_streams = false;
    int n_cus = 0;

    // descriptor ring: per set [out_ids | out_slots | in_ids | in_slots]
    int32_t *desc_host = nullptr, *desc_dev = nullptr;
    size_t desc_cap = 0;  // ints per set
    // device: [0..1] counters of stream_out's launches, [kClaimStride..+1] of stream_in's
    unsigned int *claim = nullptr;
    // ring_out[k] / ring_in[k] are recorded after the last work that reads set k
    // on each stream; they double as the end-of-work timestamps for the stats
    hipEvent_t ring_out[dkv::kRing] = {}, ring_in[dkv::kRing] = {};
    bool ring_out_rec[dkv::kRing] = {}, ring_in_rec[dkv::kRing] = {};
    int ring_cur = 0;

    dkv::Marks marks;
    dkv::Hazards hazards;
    std::vector<std::pair<int32_t, int32_t>> sort_tmp;  // (slot, id)

    // stats
    hipEvent_t ev_o0 = nullptr, ev_o1 = nullptr, ev_i0 = nullptr, ev_i1 = nullptr;
    hipEvent_t ev_join = nullptr, ev_join_in = nullptr;  // stream_out waits for stream_in / the reverse
    hipEvent_t b_o0 = nullptr, b_o1 = nullptr, b_i0 = nullptr, b_i1 = nullptr;  // this batch's first start / last end
    bool batch_open = false;
    bool out_pending = false, in_pending = false;  // work enqueued since the last kv_wait
    bool in_dirty = false;                         // stream_in holds work stream_out has not joined
    bool out_dirty = false;                        // stream_out holds work stream_in has not joined
    bool in_after_out = false;                     // block table in use: in-only work waits for earlier out work
    int n_tables = 0;                              // block tables attached (kv_destroy refuses while any is)
    // Goes up every time the engine has seen all of its enqueued work finished
    // (kv_wait, kv_query answering KV_OK, dkv::drain): what was enqueued under an
    // earlier value is done.
    uint64_t idle_epoch = 0;
    double t0 = 0;
    kv_stats acc{}, last{};
    int sticky = KV_OK;

    // Layer-wise completion of the kernel paths (cfg.chunk_layers > 0): the last
    // transfer call ran as layer_n_chunks launches of layer_chunk layers each and
    // recorded layer_ev_*[c] behind chunk c.  layer_on_out / layer_on_in say which
    // of the two event lists that call recorded (one launch for both directions
    // records on stream_out only).  layer_chunk == 0: the last call was not chunked.
    std::vector<hipEvent_t> layer_ev_out, layer_ev_in;
    int32_t layer_chunk = 0, layer_n_chunks = 0;
    bool layer_on_out = false, layer_on_in = false;

    // staging for SDMA_STAGED: one buffer per direction, chunk_cap bytes each.
    // A direction's pack / copy / unpack all run in order on that direction's
    // stream, so a buffer is never reused before its last reader is done.
    uint8_t *stage_out = nullptr, *stage_in = nullptr;
    uint64_t chunk_cap = 0;

    // synthetic decode reader
    hipStream_t s_read = nullptr;
    int32_t *read_ids = nullptr;               // device, 2 * n_hbm_blocks ints
    int32_t *read_ids_host = nullptr;          // pinned
    unsigned long long *read_acc = nullptr;    // device: [0] sum, then one 32-bit tile counter per pass
    unsigned long long *read_acc_host = nullptr;  // pinned
    std::vector<hipEvent_t> read_ev;           // passes + 1 timestamps
    int32_t read_passes = 0;
};
