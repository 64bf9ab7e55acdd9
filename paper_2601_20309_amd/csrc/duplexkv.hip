// Host side of the KV rotation engine and its C ABI (see include/duplexkv.h).
//
// Paths (how one call's bytes travel):
//   FUSED        one kv_move_kernel launch carries both directions, each lane
//                alternating an out-vector with an in-vector; zero-copy into /
//                out of the pinned pool.  Default for kv_rotate.
//   ZEROCOPY     the same kernel once per direction on the two streams.
//                Default for kv_swap_out / kv_swap_in.
//   SDMA_STAGED  pack kernel -> HBM staging -> hipMemcpyAsync per contiguous
//                host run (DMA engines), and the mirror, chunk after chunk, each
//                direction in order on its own stream.  Uses no compute units
//                for the link itself.
//   NAIVE        one hipMemcpyAsync per segment, the per-segment baseline of
//                Section 4.3.1 of the paper, kept for the benchmark ladder.
//   DMA_BLOCKS   block-first cache and block-first pool: a block is one
//                contiguous region on both sides, one hipMemcpyAsync per block
//                (the paper's "merged segments"), runs of consecutive pairs merged.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "kv_engine.hpp"
#include "kv_kernels.hpp"


namespace {

using dkv::DirDesc;
using dkv::MoveParams;

double now_ms()
{
    using clk = std::chrono::steady_clock;
    return std::chrono::duration<double, std::milli>(clk::now().time_since_epoch()).count();
}

bool config_ok(const kv_config *c)
{
    if (!c) return false;
    if (c->n_layers <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 || c->block_size <= 0 ||
        c->elem_bytes <= 0 || c->n_hbm_blocks <= 0 || c->n_host_slots <= 0)
        return false;
    if (c->host_layout != KV_HOST_BLOCK_FIRST && c->host_layout != KV_HOST_LAYER_FIRST) return false;
    if (c->path < KV_PATH_AUTO || c->path > KV_PATH_DMA_BLOCKS) return false;
    if (c->hbm_layout != KV_HBM_LAYER_FIRST && c->hbm_layout != KV_HBM_BLOCK_FIRST) return false;
    if (c->path == KV_PATH_DMA_BLOCKS &&
        (c->hbm_layout != KV_HBM_BLOCK_FIRST || c->host_layout != KV_HOST_BLOCK_FIRST))
        return false;
    if (c->chunk_layers < 0 || c->max_copy_wgs < 0) return false;
    if (c->vecs_per_lane != 0 && c->vecs_per_lane != 1 && c->vecs_per_lane != 2 && c->vecs_per_lane != 4 &&
        c->vecs_per_lane != 8)
        return false;
    if (c->wg_lanes < 0 || c->wg_lanes > dkv::kMaxThreads || c->wg_lanes % 64 != 0) return false;
    // sizes must stay far inside 64 bits
    const long double cache = 2.0L * c->n_layers * (long double)c->n_hbm_blocks * c->block_size *
                              c->n_kv_heads * c->head_dim * c->elem_bytes;
    const long double pool = 2.0L * c->n_layers * (long double)c->n_host_slots * c->block_size *
                             c->n_kv_heads * c->head_dim * c->elem_bytes;
    return cache < 1e18L && pool < 1e18L;
}

// ---- admission (host only) ------------------------------------------------
using dkv::Marks;
using dkv::kClaimStride;
using dkv::kRing;
using dkv::list_bad;

bool out_of_range(const int32_t *p, int32_t n, int32_t lim)
{
    for (int32_t i = 0; i < n; i++)
        if (p[i] < 0 || p[i] >= lim) return true;
    return false;
}

// Marks `p` with `bit`; reports a repeat inside this list and a hit on the other list.
void mark_list(std::vector<uint32_t> &m, uint32_t epoch, const int32_t *p, int32_t n, uint32_t bit,
               bool &dup, bool &overlap)
{
    for (int32_t i = 0; i < n; i++) {
        uint32_t &w = m[(size_t)p[i]];
        uint32_t bits = (w >> 2) == epoch ? (w & 3u) : 0u;
        if (bits & bit) dup = true;
        if (bits & ~bit) overlap = true;
        w = (epoch << 2) | bits | bit;
    }
}

int admit(const kv_config *c, Marks &mk, const int32_t *oi, const int32_t *os, int32_t no,
          const int32_t *ii, const int32_t *is, int32_t ni)
{
    if (list_bad(oi, no) || list_bad(os, no) || list_bad(ii, ni) || list_bad(is, ni)) return KV_EINVAL;
    if (out_of_range(oi, no, c->n_hbm_blocks) || out_of_range(ii, ni, c->n_hbm_blocks) ||
        out_of_range(os, no, c->n_host_slots) || out_of_range(is, ni, c->n_host_slots))
        return KV_ERANGE;
    mk.next();
    bool dup = false, overlap = false;
    mark_list(mk.blk, mk.epoch, oi, no, 1u, dup, overlap);
    mark_list(mk.blk, mk.epoch, ii, ni, 2u, dup, overlap);
    mark_list(mk.slot, mk.epoch, os, no, 1u, dup, overlap);
    mark_list(mk.slot, mk.epoch, is, ni, 2u, dup, overlap);
    if (dup) return KV_EDUP;
    if (overlap) return KV_EOVERLAP;
    return KV_OK;
}

}  // namespace


namespace {

#define HIPTRY(e, call)                                                                      \
    do {                                                                                     \
        hipError_t err_ = (call);                                                            \
        if (err_ != hipSuccess) {                                                            \
            fprintf(stderr, "duplexkv: %s failed: %s (%s:%d)\n", #call, hipGetErrorString(err_), \
                    __FILE__, __LINE__);                                                     \
            if (e) (e)->sticky = KV_EHIP;                                                    \
            return KV_EHIP;                                                                  \
        }                                                                                    \
    } while (0)

uint64_t seg_of(const kv_config *c)
{
    return (uint64_t)c->block_size * (uint64_t)c->n_kv_heads * (uint64_t)c->head_dim *
           (uint64_t)c->elem_bytes;
}

int pick_vec(const kv_engine *e)
{
    const uint64_t a = (uint64_t)(uintptr_t)e->hbm | (uint64_t)(uintptr_t)e->pool | e->seg;
    for (int v = 16; v > 1; v >>= 1)
        if ((a & (uint64_t)(v - 1)) == 0) return v;
    return 1;
}

// The four id arrays of a launch (device pointers; a direction that is not
// used, or whose slots are the list indices, passes nullptr).
struct MoveIds {
    const int32_t *out_ids, *out_slots, *in_ids, *in_slots;
};

// `wgs` workgroups of `lanes` lanes; the waves among them are the workers, and
// no more of them are launched than the launch has steps.
template <int U, bool LINK>
void launch_move_v(int vec, int wgs, int lanes, hipStream_t s, const MoveParams &p, const MoveIds &d)
{
    const uint32_t steps = p.mix_q ? p.in.tiles : std::max(p.out.tiles, p.in.tiles);
    const uint32_t waves_per_wg = (uint32_t)lanes / dkv::kWave;
    wgs = (int)std::max<uint32_t>(1u, std::min<uint32_t>((uint32_t)wgs, (steps + waves_per_wg - 1) / waves_per_wg));
    dim3 g((unsigned)wgs), b((unsigned)lanes);
#define DKV_LAUNCH(V) \
    hipLaunchKernelGGL((dkv::kv_move_kernel<V, U, LINK>), g, b, 0, s, p, d.out_ids, d.out_slots, d.in_ids, d.in_slots)
    switch (vec) {
    case 16: DKV_LAUNCH(dkv::u32x4); break;
    case 8: DKV_LAUNCH(dkv::u32x2); break;
    case 4: DKV_LAUNCH(unsigned int); break;
    case 2: DKV_LAUNCH(unsigned short); break;
    default: DKV_LAUNCH(unsigned char); break;
    }
#undef DKV_LAUNCH
}

// link: the far side is host memory (zero-copy paths); else HBM staging.
void launch_move(int u, int vec, int wgs, int lanes, hipStream_t s, const MoveParams &p, const MoveIds &d, bool link)
{
    if (link) {
        switch (u) {
        case 1: launch_move_v<1, true>(vec, wgs, lanes, s, p, d); break;
        case 2: launch_move_v<2, true>(vec, wgs, lanes, s, p, d); break;
        case 4: launch_move_v<4, true>(vec, wgs, lanes, s, p, d); break;
        default: launch_move_v<8, true>(vec, wgs, lanes, s, p, d); break;
        }
    } else {
        switch (u) {
        case 1: launch_move_v<1, false>(vec, wgs, lanes, s, p, d); break;
        case 2: launch_move_v<2, false>(vec, wgs, lanes, s, p, d); break;
        case 4: launch_move_v<4, false>(vec, wgs, lanes, s, p, d); break;
        default: launch_move_v<8, false>(vec, wgs, lanes, s, p, d); break;
        }
    }
}

void hbm_strides(const kv_engine *e, uint64_t &plane_stride, uint64_t &block_stride)
{
    if (e->cfg.hbm_layout == KV_HBM_BLOCK_FIRST) {
        plane_stride = e->seg;
        block_stride = (uint64_t)e->n_planes * e->seg;
    } else {
        plane_stride = (uint64_t)e->cfg.n_hbm_blocks * e->seg;
        block_stride = e->seg;
    }
}

// Fills the fields common to every launch; `u` = vectors per lane per tile.
MoveParams base_params(const kv_engine *e, int u)
{
    MoveParams p{};
    p.hbm = e->hbm;
    p.seg_bytes = e->seg;
    hbm_strides(e, p.hbm_plane_stride, p.hbm_block_stride);
    p.plane0 = 0;
    p.n_planes = e->n_planes;
    p.vec_per_seg = (uint32_t)(e->seg / (uint64_t)e->vec);
    const uint32_t tile = (uint32_t)dkv::kWave * (uint32_t)u;
    p.tiles_per_seg = (p.vec_per_seg + tile - 1) / tile;
    p.full_tiles = p.vec_per_seg % tile == 0 ? 1u : 0u;
    return p;
}

void pool_strides(const kv_engine *e, uint64_t &slot_stride, uint64_t &plane_stride)
{
    if (e->cfg.host_layout == KV_HOST_BLOCK_FIRST) {
        slot_stride = (uint64_t)e->n_planes * e->seg;
        plane_stride = e->seg;
    } else {
        slot_stride = e->seg;
        plane_stride = (uint64_t)e->cfg.n_host_slots * e->seg;
    }
}

// tiles of one direction over `planes` planes; false if the count leaves no
// headroom in 32 bits (the kernels step a tile index by the grid size)
bool dir_tiles(uint32_t n, uint32_t planes, uint32_t tiles_per_seg, uint32_t &tiles)
{
    const uint64_t t = (uint64_t)n * planes * tiles_per_seg;
    if (t >= 0x7FFFFFFFull) return false;
    tiles = (uint32_t)t;
    return true;
}

int acquire_ring(kv_engine *e, int &k)
{
    k = e->ring_cur;
    e->ring_cur = (e->ring_cur + 1) % kRing;
    // set still referenced by enqueued work: let it drain
    if (e->ring_out_rec[k]) HIPTRY(e, hipEventSynchronize(e->ring_out[k]));
    if (e->ring_in_rec[k]) HIPTRY(e, hipEventSynchronize(e->ring_in[k]));
    e->ring_out_rec[k] = e->ring_in_rec[k] = false;
    return KV_OK;
}

void open_batch(kv_engine *e)
{
    if (!e->batch_open) {
        e->batch_open = true;
        e->b_o0 = e->b_o1 = e->b_i0 = e->b_i1 = nullptr;
        e->t0 = now_ms();
        e->acc = kv_stats{};
    }
}

// First work of a direction in this batch: timestamp its start on stream s.
int mark_start(kv_engine *e, bool out_side, hipStream_t s)
{
    if (out_side && !e->b_o0) {
        HIPTRY(e, hipEventRecord(e->ev_o0, s));
        e->b_o0 = e->ev_o0;
    }
    if (!out_side && !e->b_i0) {
        HIPTRY(e, hipEventRecord(e->ev_i0, s));
        e->b_i0 = e->ev_i0;
    }
    return KV_OK;
}

// Last work of a direction in this call: releases descriptor set k and is the
// end timestamp so far.
int mark_end(kv_engine *e, bool out_side, int k, hipStream_t s)
{
    if (out_side) {
        HIPTRY(e, hipEventRecord(e->ring_out[k], s));
        e->ring_out_rec[k] = true;
        e->b_o1 = e->ring_out[k];
        e->out_pending = true;
        e->out_dirty = true;
    } else {
        HIPTRY(e, hipEventRecord(e->ring_in[k], s));
        e->ring_in_rec[k] = true;
        e->b_i1 = e->ring_in[k];
        e->in_pending = true;
        e->in_dirty = true;
    }
    return KV_OK;
}

// Launch shape of a link-bound kernel: workgroups, lanes per workgroup, vectors
// per lane per tile.  Waves are the workers, each with one tile (U KiB per
// direction at 16-byte vectors) in flight; workgroups only pack them.  What
// saturates PCIe Gen5 x16 is bytes in flight; what a kernel running beside the
// copy loses grows with the number of copy waves, steeply once the copy issues
// more than the link drains.  So each kind of launch gets the smallest shape
// that holds its rate both alone and beside an HBM-bound reader (measured,
// scattered 2 MiB blocks, 4 GiB per direction; GB/s alone / beside the reader,
// and what the reader keeps of its 6.5 TB/s):
//  both directions in one launch, U = 1:
//     80 waves  97.5 /  83.5 (5.59)     112 waves 100.7 /  99.9 (5.30)
//     96 waves 100.2 /  96.4 (5.45)     144 waves 100.8 / 100.6 (4.94)
//    (32 waves x U 4: 100.1 / 99.2 (5.52), but 99.4 instead of 100.1 at 256 MiB)
//  swap-out alone: host-bound stores are paced by nothing but the link, and
//  every wave beyond those that fill it only gets in the reader's way:
//     U 1:  48 waves 56.7 / 46.6 (5.99)   64 waves 56.5 / 56.7 (5.34)   112 waves 55.8 / 56.8 (3.00)
//     U 4:  16 waves 56.8 / 56.7 (5.68)   20 waves 56.7 / 56.8 (4.69)    24 waves 56.4 / 56.8 (3.75)
//     U 8:  10 waves 56.7 / 51.0 (6.34)   12 waves 56.7 / 56.7 (5.93)
//  swap-in alone:
//     U 1:  64 waves 49.3 / 48.3 (5.49)   80 waves 57.4 / 56.8 (5.30)   112 waves 57.5 / 57.4 (4.88)
//     U 4:  20 waves 55.2 / 54.2 (5.53)   24 waves 57.5 / 57.2 (5.44)
//     U 8:  14 waves 57.5 / 51.3 (5.45)   16 waves 57.5 / 55.6 (5.36)
//  both directions in one launch with at least twice as much coming in as
//  going out (the usual rotation once eager copies have run): the rate is the
//  swap-in's, and 32 waves x U 4 hold it (out : in blocks, GB/s summed alone /
//  beside the reader, reader):
//     8 : 2048   112 x 1  57.4 / 57.3 (4.87)    32 x 4  57.5 / 57.3 (5.36)
//  1024 : 2048   112 x 1  85.8 / 85.2 (5.09)    32 x 4  85.9 / 85.2 (5.38)
//  1536 : 2048   112 x 1 100.1 / 98.8 (5.20)    32 x 4  99.6 / 97.9 (5.40)   (not taken: 112 x 1 stays)
// The same waves packed four or sixteen to a workgroup do no better.
// A configured vecs_per_lane is kept (the wave count follows it); max_copy_wgs
// counts workgroups of wg_lanes lanes and set alone keeps 256-lane workgroups;
// wg_lanes set alone keeps the number of waves.
enum LinkKind { kBoth, kInHeavy, kOutOnly, kInOnly };
struct LinkShape { int wgs, lanes, u; };

LinkShape link_shape(const kv_engine *e, LinkKind kind)
{
    const int cw = e->cfg.max_copy_wgs, cl = e->cfg.wg_lanes, cu = e->cfg.vecs_per_lane;
    int u = cu ? cu : (kind == kOutOnly ? 8 : kind == kInOnly || kind == kInHeavy ? 4 : 1);
    if (!cu) {  // whole tiles only: the segment must be a multiple of the tile
        const uint64_t vec_per_seg = e->seg / (uint64_t)e->vec;
        while (u > 1 && vec_per_seg % ((uint64_t)dkv::kWave * (uint64_t)u) != 0) u >>= 1;
    }
    int waves;
    switch (kind) {
    case kOutOnly: waves = u >= 8 ? 12 : u == 4 ? 16 : u == 2 ? 32 : 64; break;
    case kInOnly: waves = u >= 8 ? 16 : u == 4 ? 24 : u == 2 ? 44 : 80; break;
    default: waves = u >= 8 ? 20 : u == 4 ? 32 : u == 2 ? 64 : 112; break;  // kBoth and kInHeavy differ in u
    }
    LinkShape s;
    s.u = u;
    s.lanes = cl ? cl : (cw ? dkv::kThreads : dkv::kWave);
    s.wgs = cw ? cw : std::max(1, waves * dkv::kWave / s.lanes);
    return s;
}

// HBM-bound pack / unpack launches.  Measured on one 256 MiB chunk of scattered
// 32 KiB segments (bare kernel time, source in no cache): persistent waves that
// loop over 4 KiB tiles, 2048 workgroups, 93 us; one 4 KiB tile per wave (16384
// workgroups) 89 us; one 1 KiB tile per wave and no loop at all (65536
// workgroups of 4 waves, dealt out by the hardware dispatcher) 86 us = 78 % of
// the HBM peak, against 100 us for the runtime's own device copy of that size.
// The general move kernel pays too much per wave for tiles that small, so this
// shape has a kernel of its own (kv_stage_kernel).  A configured max_copy_wgs (a
// copy that has to stay small beside other kernels) keeps that many persistent
// workgroups of the move kernel with 4 KiB tiles.
template <bool UNPACK>
void launch_stage(int vec, hipStream_t s, const dkv::StageParams &p, const int32_t *ids)
{
    // four waves to a workgroup for the gather, one for the scatter (see kv_stage_kernel)
    const uint32_t waves_per_wg = UNPACK ? 1u : dkv::kThreads / dkv::kWave;
    dim3 g((p.tiles + waves_per_wg - 1) / waves_per_wg), b(waves_per_wg * dkv::kWave);
#define DKV_STAGE(V) hipLaunchKernelGGL((dkv::kv_stage_kernel<V, UNPACK>), g, b, 0, s, p, ids)
    switch (vec) {
    case 16: DKV_STAGE(dkv::u32x4); break;
    case 8: DKV_STAGE(dkv::u32x2); break;
    case 4: DKV_STAGE(unsigned int); break;
    case 2: DKV_STAGE(unsigned short); break;
    default: DKV_STAGE(unsigned char); break;
    }
#undef DKV_STAGE
}

// ---- FUSED / ZEROCOPY -----------------------------------------------------
// One link-bound launch, or, with cfg.chunk_layers set, one launch per chunk of
// that many layers, lowest layers first, each followed by an event in `ev`, so
// that whoever consumes the blocks (the model's layer l, a writer of the pool)
// can start on a layer while the later ones still move.  A chunk is the same
// kernel over planes [p0, p1) of every block of the call.
int launch_link(kv_engine *e, const LinkShape &sh, hipStream_t s, const MoveParams &whole, const MoveIds &ids,
                std::vector<hipEvent_t> *ev)
{
    const uint32_t per_chunk = ev ? 2u * (uint32_t)e->cfg.chunk_layers : whole.n_planes;
    uint32_t c = 0;
    for (uint32_t p0 = 0; p0 < whole.n_planes; p0 += per_chunk, c++) {
        MoveParams q = whole;
        q.plane0 = p0;
        q.n_planes = std::min(per_chunk, whole.n_planes - p0);
        q.out.tiles = q.out.n * q.n_planes * q.tiles_per_seg;  // fits: the whole call's count was checked
        q.in.tiles = q.in.n * q.n_planes * q.tiles_per_seg;
        q.mix_q = whole.mix_q && q.out.tiles ? (((uint64_t)q.out.tiles << 32) + q.in.tiles - 1) / q.in.tiles : 0;
        launch_move(sh.u, e->vec, sh.wgs, sh.lanes, s, q, ids, true);
        HIPTRY(e, hipGetLastError());
        e->acc.n_launches += 1;
        if (ev) HIPTRY(e, hipEventRecord((*ev)[c], s));
    }
    return KV_OK;
}

int run_zero_copy(kv_engine *e, int path, int k, int32_t no, int32_t ni)
{
    int32_t *dh = e->desc_host + (size_t)k * e->desc_cap;
    const bool fused = path == KV_PATH_FUSED && no > 0 && ni > 0;
    auto params = [&](int u, unsigned int *claim) {
        MoveParams q = base_params(e, u);
        q.claim = claim;
        q.far_out = e->pool;
        q.far_in = e->pool;
        pool_strides(e, q.far_slot_stride_out, q.far_plane_stride_out);
        q.far_slot_stride_in = q.far_slot_stride_out;
        q.far_plane_stride_in = q.far_plane_stride_out;
        q.plane_major = e->cfg.host_layout == KV_HOST_LAYER_FIRST ? 1u : 0u;
        return q;
    };
    // The link-bound kernels fetch ids and slots with scalar loads.  Where one list
    // entry stands for many tiles (a whole block in block-first pool order) they
    // read the pinned ring in place: a few thousand 64-byte reads over a link that
    // moves gigabytes, no upload, nothing between the call and the launch.  Where
    // an entry stands for little (small segments, few layers, or plane-major
    // order, in which every segment is its own visit) every workgroup fetches a
    // new entry nearly every tile; those reads would then be an eighth of the
    // link traffic (4 KiB segments, one layer: 83 instead of 93 GB/s), so the set
    // is uploaded first, ~5 us on the launch's stream.
    const uint64_t visit_bytes = e->cfg.host_layout == KV_HOST_LAYER_FIRST ? e->seg : e->block_bytes;
    const bool upload = visit_bytes < (256u << 10);
    int32_t *dd = upload ? e->desc_dev + (size_t)k * e->desc_cap : dh;
    int32_t *d_o = dd, *d_i = dd + 2 * (size_t)no;  // each: [ids | slots]
    auto upload_ids = [&](bool out_part, bool in_part, hipStream_t s) -> int {
        if (!upload) return KV_OK;
        const size_t a = out_part ? 0 : 2 * (size_t)no, b = in_part ? 2 * ((size_t)no + ni) : 2 * (size_t)no;
        HIPTRY(e, hipMemcpyAsync(dd + a, dh + a, (b - a) * sizeof(int32_t), hipMemcpyHostToDevice, s));
        return KV_OK;
    };
    const DirDesc none{0, 0, 0, 0};
    auto desc = [](const MoveParams &q, int32_t n, DirDesc &d) {
        d = DirDesc{(uint32_t)n, 0, 0, 0};
        return dir_tiles((uint32_t)n, q.n_planes, q.tiles_per_seg, d.tiles);
    };

    if (fused) {
        // one launch on stream_out carries both directions; stream_in is joined
        // before (if it holds work) and after
        const LinkShape sh = link_shape(e, ni >= 2 * (int64_t)no ? kInHeavy : kBoth);
        // What the out list has beyond the in list is a swap-out on its own: from
        // kSplitBytes on it gets the launch shape of one (12 waves instead of 112:
        // 56.7 against 55.8 GB/s, and a co-runner keeps 5.9 instead of 3.0 TB/s),
        // right behind the paired part on the same stream.
        constexpr uint64_t kSplitBytes = 64ull << 20;
        const bool layered = e->cfg.chunk_layers > 0;  // layer by layer: the whole out list stays in the one kernel
        const int32_t n_rest =
            !layered && no > ni && (uint64_t)(no - ni) * e->block_bytes >= kSplitBytes ? no - ni : 0;
        const int32_t no_paired = no - n_rest;
        const LinkShape sh_rest = link_shape(e, kOutOnly);
        MoveParams p = params(sh.u, e->claim), p_rest = params(sh_rest.u, e->claim);
        p_rest.in = none;
        if (!desc(p, no_paired, p.out) || !desc(p, ni, p.in) || !desc(p_rest, n_rest, p_rest.out)) return KV_EUNSUP;
        // in list longer: spread the out tiles over it instead of pairing 1:1
        if (p.in.tiles > p.out.tiles)
            p.mix_q = (((uint64_t)p.out.tiles << 32) + p.in.tiles - 1) / p.in.tiles;
        if (e->in_dirty || !e->own_streams) {
            HIPTRY(e, hipEventRecord(e->ev_join, e->s_in));
            HIPTRY(e, hipStreamWaitEvent(e->s_out, e->ev_join, 0));
            e->in_dirty = false;
        }
        if (upload_ids(true, true, e->s_out) != KV_OK) return KV_EHIP;
        if (!e->b_o0 && !e->b_i0) {  // one start timestamp serves both directions
            if (mark_start(e, true, e->s_out) != KV_OK) return KV_EHIP;
            e->b_i0 = e->b_o0;
        } else {
            if (mark_start(e, true, e->s_out) != KV_OK) return KV_EHIP;
            if (!e->b_i0) {
                HIPTRY(e, hipEventRecord(e->ev_i0, e->s_out));
                e->b_i0 = e->ev_i0;
            }
        }
        if (launch_link(e, sh, e->s_out, p, MoveIds{d_o, d_o + no, d_i, d_i + ni},
                        layered ? &e->layer_ev_out : nullptr) != KV_OK)
            return KV_EHIP;
        e->layer_chunk = layered ? e->cfg.chunk_layers : 0;
        e->layer_on_out = layered;
        e->layer_on_in = false;
        if (n_rest > 0) {
            launch_move(sh_rest.u, e->vec, sh_rest.wgs, sh_rest.lanes, e->s_out, p_rest,
                        MoveIds{d_o + no_paired, d_o + no + no_paired, nullptr, nullptr}, true);
            HIPTRY(e, hipGetLastError());
            e->acc.n_launches += 1;
        }
        if (mark_end(e, true, k, e->s_out) != KV_OK) return KV_EHIP;
        e->b_i1 = e->ring_out[k];
        HIPTRY(e, hipStreamWaitEvent(e->s_in, e->ring_out[k], 0));
        e->out_dirty = false;
        return KV_OK;
    }
    // One kernel per direction, each on its own stream.  When both run at once
    // they only reach the rate of the fused launch if each has at least one
    // workgroup per CU (measured, one-wave workgroups per kernel, U = 1, 256 + 256
    // MiB: 112 -> 70, 192 -> 77, 240 -> 87, 256 -> 99.9, 288 -> 99.5, 384 -> 98.5
    // GB/s; the same 256 waves packed as 64 x 256 lanes -> 76).
    LinkShape sh_out = link_shape(e, kOutOnly), sh_in = link_shape(e, kInOnly);
    if (no > 0 && ni > 0 && !e->cfg.max_copy_wgs && !e->cfg.wg_lanes && !e->cfg.vecs_per_lane) {
        sh_out.wgs = sh_in.wgs = 9 * (e->n_cus > 0 ? e->n_cus : 256) / 8;
        sh_out.lanes = sh_in.lanes = dkv::kWave;
        sh_out.u = sh_in.u = 1;
    }
    const MoveIds ids_out{d_o, d_o + no, nullptr, nullptr}, ids_in{nullptr, nullptr, d_i, d_i + ni};
    // launches on stream_out draw from the first pair of counters, those on stream_in from the second
    MoveParams p_out = params(sh_out.u, e->claim), p_in = params(sh_in.u, e->claim + kClaimStride);
    p_out.in = p_in.out = none;
    if (!desc(p_out, no, p_out.out) || !desc(p_in, ni, p_in.in)) return KV_EUNSUP;  // before anything is enqueued
    // The block table promises that no block or slot is overwritten while an
    // earlier transfer still reads it, and none read while an earlier one still
    // writes it.  Its lists are conflict-free within a call but reuse, across
    // calls, what earlier calls vacated; so each direction of a call first waits
    // for what the other stream was given before this call, whether or not the
    // call carries the other direction too (its own two directions still run
    // side by side).
    if (e->in_after_out && no > 0 && e->in_dirty) {
        // a block this copy-out reads may still be being written by an earlier swap-in
        HIPTRY(e, hipEventRecord(e->ev_join, e->s_in));
        HIPTRY(e, hipStreamWaitEvent(e->s_out, e->ev_join, 0));
        e->in_dirty = false;
    }
    if (e->in_after_out && ni > 0 && e->out_dirty) {
        // a block or slot this swap-in overwrites may still be read by an earlier copy-out
        HIPTRY(e, hipEventRecord(e->ev_join_in, e->s_out));
        HIPTRY(e, hipStreamWaitEvent(e->s_in, e->ev_join_in, 0));
        e->out_dirty = false;
    }
    const bool layered = e->cfg.chunk_layers > 0;
    e->layer_chunk = layered ? e->cfg.chunk_layers : 0;
    e->layer_on_out = layered && no > 0;
    e->layer_on_in = layered && ni > 0;
    if (no > 0) {
        if (upload_ids(true, false, e->s_out) != KV_OK) return KV_EHIP;
        if (mark_start(e, true, e->s_out) != KV_OK) return KV_EHIP;
        if (launch_link(e, sh_out, e->s_out, p_out, ids_out, layered ? &e->layer_ev_out : nullptr) != KV_OK)
            return KV_EHIP;
        if (mark_end(e, true, k, e->s_out) != KV_OK) return KV_EHIP;
    }
    if (ni > 0) {
        if (upload_ids(false, true, e->s_in) != KV_OK) return KV_EHIP;
        if (mark_start(e, false, e->s_in) != KV_OK) return KV_EHIP;
        if (launch_link(e, sh_in, e->s_in, p_in, ids_in, layered ? &e->layer_ev_in : nullptr) != KV_OK)
            return KV_EHIP;
        if (mark_end(e, false, k, e->s_in) != KV_OK) return KV_EHIP;
    }
    return KV_OK;
}

// ---- NAIVE: one copy per segment -------------------------------------------
int run_naive(kv_engine *e, const int32_t *oi, const int32_t *os, int32_t no, const int32_t *ii,
              const int32_t *is, int32_t ni)
{
    uint64_t ss, ps;
    pool_strides(e, ss, ps);
    uint64_t hps, hbs;
    hbm_strides(e, hps, hbs);
    if (no > 0 && mark_start(e, true, e->s_out) != KV_OK) return KV_EHIP;
    if (ni > 0 && mark_start(e, false, e->s_in) != KV_OK) return KV_EHIP;
    const int32_t nmax = std::max(no, ni);
    for (int32_t i = 0; i < nmax; i++) {  // interleave so both streams fill together
        for (uint32_t pl = 0; pl < e->n_planes; pl++) {
            if (i < no) {
                HIPTRY(e, hipMemcpyAsync(e->pool + (uint64_t)os[i] * ss + pl * ps,
                                         e->hbm + pl * hps + (uint64_t)oi[i] * hbs, e->seg,
                                         hipMemcpyDeviceToHost, e->s_out));
            }
            if (i < ni) {
                HIPTRY(e, hipMemcpyAsync(e->hbm + pl * hps + (uint64_t)ii[i] * hbs,
                                         e->pool + (uint64_t)is[i] * ss + pl * ps, e->seg,
                                         hipMemcpyHostToDevice, e->s_in));
            }
        }
    }
    e->acc.n_launches += (int32_t)(((int64_t)no + ni) * e->n_planes);
    if (no > 0) {
        HIPTRY(e, hipEventRecord(e->ev_o1, e->s_out));
        e->b_o1 = e->ev_o1;
        e->out_pending = e->out_dirty = true;
    }
    if (ni > 0) {
        HIPTRY(e, hipEventRecord(e->ev_i1, e->s_in));
        e->b_i1 = e->ev_i1;
        e->in_pending = e->in_dirty = true;
    }
    return KV_OK;
}

// ---- DMA_BLOCKS: one copy per block, both sides block-first -----------------------
int run_dma_blocks(kv_engine *e, const int32_t *oi, const int32_t *os, int32_t no, const int32_t *ii,
                   const int32_t *is, int32_t ni)
{
    const uint64_t bb = e->block_bytes;
    if (no > 0 && mark_start(e, true, e->s_out) != KV_OK) return KV_EHIP;
    if (ni > 0 && mark_start(e, false, e->s_in) != KV_OK) return KV_EHIP;
    int32_t a = 0, b = 0, n_copies = 0;
    while (a < no || b < ni) {  // alternate so both streams fill together
        if (a < no) {
            int32_t r = a + 1;  // run in which block ids and slots both advance by one
            while (r < no && oi[r] == oi[r - 1] + 1 && os[r] == os[r - 1] + 1) r++;
            HIPTRY(e, hipMemcpyAsync(e->pool + (uint64_t)os[a] * bb, e->hbm + (uint64_t)oi[a] * bb,
                                     (uint64_t)(r - a) * bb, hipMemcpyDeviceToHost, e->s_out));
            a = r;
            n_copies++;
        }
        if (b < ni) {
            int32_t r = b + 1;
            while (r < ni && ii[r] == ii[r - 1] + 1 && is[r] == is[r - 1] + 1) r++;
            HIPTRY(e, hipMemcpyAsync(e->hbm + (uint64_t)ii[b] * bb, e->pool + (uint64_t)is[b] * bb,
                                     (uint64_t)(r - b) * bb, hipMemcpyHostToDevice, e->s_in));
            b = r;
            n_copies++;
        }
    }
    e->acc.n_launches += n_copies;
    if (no > 0) {
        HIPTRY(e, hipEventRecord(e->ev_o1, e->s_out));
        e->b_o1 = e->ev_o1;
        e->out_pending = e->out_dirty = true;
    }
    if (ni > 0) {
        HIPTRY(e, hipEventRecord(e->ev_i1, e->s_in));
        e->b_i1 = e->ev_i1;
        e->in_pending = e->in_dirty = true;
    }
    return KV_OK;
}

// ---- SDMA_STAGED -----------------------------------------------------------
// A chunk is blocks [j0, j1) of the slot-sorted list x planes [p0, p1).  Its
// staging image mirrors the host layout ([j][plane][seg] for block-first,
// [plane][j][seg] for layer-first) so that every run of consecutive slots is
// one contiguous range on both sides and costs one DMA copy.
struct ChunkPlan {
    uint32_t blocks_per_chunk, planes_per_chunk;
};

int plan_chunks(const kv_engine *e, uint32_t n, ChunkPlan &pl)
{
    const uint64_t cap = e->chunk_cap;
    if (e->cfg.host_layout == KV_HOST_BLOCK_FIRST) {
        uint32_t planes = e->cfg.chunk_layers > 0 ? std::min<uint32_t>(2u * e->cfg.chunk_layers, e->n_planes)
                                                 : e->n_planes;
        while (planes > 2 && (uint64_t)planes * e->seg > cap) planes -= 2;
        if ((uint64_t)planes * e->seg > cap) return KV_EUNSUP;
        pl.planes_per_chunk = planes;
        pl.blocks_per_chunk = (uint32_t)std::min<uint64_t>(n, cap / ((uint64_t)planes * e->seg));
    } else {
        uint32_t blocks = n;
        if (2ull * blocks * e->seg > cap) blocks = (uint32_t)(cap / (2ull * e->seg));
        if (blocks == 0) return KV_EUNSUP;
        uint32_t layers = (uint32_t)std::min<uint64_t>((uint64_t)e->cfg.n_layers,
                                                        cap / (2ull * blocks * e->seg));
        if (e->cfg.chunk_layers > 0) layers = std::min<uint32_t>(layers, (uint32_t)e->cfg.chunk_layers);
        pl.blocks_per_chunk = blocks;
        pl.planes_per_chunk = 2 * std::max(layers, 1u);
    }
    return KV_OK;
}

// Sorts (slot, id) pairs by slot into the descriptor set: ids at dst[0..n), slots at dst[n..2n).
void sorted_desc(kv_engine *e, const int32_t *ids, const int32_t *slots, int32_t n, int32_t *dst)
{
    e->sort_tmp.resize((size_t)n);
    for (int32_t i = 0; i < n; i++) e->sort_tmp[(size_t)i] = {slots[i], ids[i]};
    std::sort(e->sort_tmp.begin(), e->sort_tmp.end());
    for (int32_t i = 0; i < n; i++) {
        dst[i] = e->sort_tmp[(size_t)i].second;
        dst[(size_t)n + i] = e->sort_tmp[(size_t)i].first;
    }
}

// Copies of one chunk between staging and pool.  `to_host` picks the direction.
int chunk_copies(kv_engine *e, bool to_host, uint8_t *stage, const int32_t *sorted_slots, uint32_t j0,
                 uint32_t j1, uint32_t p0, uint32_t p1, hipStream_t s, int32_t &n_copies)
{
    const uint32_t nb = j1 - j0, np = p1 - p0;
    uint64_t ss, ps;
    pool_strides(e, ss, ps);
    auto copy = [&](uint64_t pool_off, uint64_t stage_off, uint64_t bytes) -> hipError_t {
        n_copies++;
        return to_host ? hipMemcpyAsync(e->pool + pool_off, stage + stage_off, bytes, hipMemcpyDeviceToHost, s)
                       : hipMemcpyAsync(stage + stage_off, e->pool + pool_off, bytes, hipMemcpyHostToDevice, s);
    };
    const bool block_first = e->cfg.host_layout == KV_HOST_BLOCK_FIRST;
    uint32_t j = j0;
    while (j < j1) {  // run of consecutive slots [j, r)
        uint32_t r = j + 1;
        while (r < j1 && sorted_slots[r] == sorted_slots[r - 1] + 1) r++;
        const uint64_t slot = (uint64_t)sorted_slots[j];
        if (block_first) {
            if (np == e->n_planes) {  // whole blocks: the run is one range
                HIPTRY(e, copy(slot * ss, (uint64_t)(j - j0) * np * e->seg, (uint64_t)(r - j) * np * e->seg));
            } else {
                for (uint32_t b = j; b < r; b++)
                    HIPTRY(e, copy((uint64_t)sorted_slots[b] * ss + (uint64_t)p0 * ps,
                                   (uint64_t)(b - j0) * np * e->seg, (uint64_t)np * e->seg));
            }
        } else {
            for (uint32_t pl = p0; pl < p1; pl++)
                HIPTRY(e, copy(slot * ss + (uint64_t)pl * ps,
                               ((uint64_t)(pl - p0) * nb + (j - j0)) * e->seg, (uint64_t)(r - j) * e->seg));
        }
        j = r;
    }
    return KV_OK;
}

MoveParams stage_params(const kv_engine *e, uint8_t *stage, uint32_t nb, uint32_t p0, uint32_t np, int u)
{
    MoveParams p = base_params(e, u);
    p.plane0 = p0;
    p.n_planes = np;
    p.far_out = p.far_in = stage;
    uint64_t ss, ps;
    if (e->cfg.host_layout == KV_HOST_BLOCK_FIRST) {
        ss = (uint64_t)np * e->seg;
        ps = e->seg;
        p.plane_major = 0;
    } else {
        ss = e->seg;
        ps = (uint64_t)nb * e->seg;
        p.plane_major = 1;
    }
    // the kernel adds plane * ps with the absolute plane index: rebase to p0
    p.far_out = p.far_in = stage - (uint64_t)p0 * ps;
    p.far_slot_stride_out = p.far_slot_stride_in = ss;
    p.far_plane_stride_out = p.far_plane_stride_in = ps;
    return p;
}

// The same chunk for kv_stage_kernel; false if it has too many tiles for a 32-bit index.
bool stage_kernel_params(const kv_engine *e, uint8_t *stage, uint32_t nb, uint32_t p0, uint32_t np,
                         dkv::StageParams &q)
{
    q = dkv::StageParams{};
    q.hbm = e->hbm;
    q.stage = stage;
    hbm_strides(e, q.hbm_plane_stride, q.hbm_block_stride);
    if (e->cfg.host_layout == KV_HOST_BLOCK_FIRST) {
        q.slot_stride = (uint64_t)np * e->seg;
        q.plane_stride = e->seg;
        q.plane_major = 0;
    } else {
        q.slot_stride = e->seg;
        q.plane_stride = (uint64_t)nb * e->seg;
        q.plane_major = 1;
    }
    q.plane0 = p0;
    q.n_planes = np;
    q.n = nb;
    q.vec_per_seg = (uint32_t)(e->seg / (uint64_t)e->vec);
    q.tiles_per_seg = (q.vec_per_seg + dkv::kWave - 1) / dkv::kWave;
    return dir_tiles(nb, np, q.tiles_per_seg, q.tiles);
}

int run_staged(kv_engine *e, int k, const int32_t *oi, const int32_t *os, int32_t no, const int32_t *ii,
               const int32_t *is, int32_t ni)
{
    int32_t *dh = e->desc_host + (size_t)k * e->desc_cap;
    int32_t *dd = e->desc_dev + (size_t)k * e->desc_cap;
    int32_t *h_out = dh, *h_in = dh + 2 * (size_t)no;
    int32_t *d_out = dd, *d_in = dd + 2 * (size_t)no;
    constexpr int U = 4;                         // capped launches: persistent waves, 4 KiB tiles
    const int cap_wgs = e->cfg.max_copy_wgs;     // 0: one wave per 1 KiB tile, kv_stage_kernel
    ChunkPlan po{}, pi{};
    if (no > 0) {
        int rc = plan_chunks(e, (uint32_t)no, po);
        if (rc != KV_OK) return rc;
        sorted_desc(e, oi, os, no, h_out);
    }
    if (ni > 0) {
        int rc = plan_chunks(e, (uint32_t)ni, pi);
        if (rc != KV_OK) return rc;
        sorted_desc(e, ii, is, ni, h_in);
    }
    // every chunk's tile count must fit the kernels' 32-bit index: checked for the
    // largest chunk of each direction before anything is enqueued
    {
        const uint64_t vec_per_seg = e->seg / (uint64_t)e->vec;
        const uint64_t tile = (uint64_t)dkv::kWave * (cap_wgs > 0 ? U : 1);
        const uint32_t tiles_per_seg = (uint32_t)((vec_per_seg + tile - 1) / tile);
        uint32_t unused;
        if ((no > 0 && !dir_tiles(po.blocks_per_chunk, po.planes_per_chunk, tiles_per_seg, unused)) ||
            (ni > 0 && !dir_tiles(pi.blocks_per_chunk, pi.planes_per_chunk, tiles_per_seg, unused)))
            return KV_EUNSUP;
    }
    if (no > 0) {
        HIPTRY(e, hipMemcpyAsync(d_out, h_out, 2 * (size_t)no * sizeof(int32_t), hipMemcpyHostToDevice, e->s_out));
        if (mark_start(e, true, e->s_out) != KV_OK) return KV_EHIP;
    }
    if (ni > 0) {
        HIPTRY(e, hipMemcpyAsync(d_in, h_in, 2 * (size_t)ni * sizeof(int32_t), hipMemcpyHostToDevice, e->s_in));
        if (mark_start(e, false, e->s_in) != KV_OK) return KV_EHIP;
    }
    // Chunks of the two directions are enqueued alternately so both streams fill
    // together.  out: pack(c) then its copies; in: copies of c then unpack(c).
    struct Cur { uint32_t j0 = 0, p0 = 0; bool done = true; } co, ci;
    co.done = no == 0;
    ci.done = ni == 0;
    int32_t n_ops = 0;
    // Layer by layer for a consumer (kv_stream_wait_layer): possible when a chunk is
    // chunk_layers layers of the whole list, i.e. the staging buffer did not force
    // the list or the chunk to be cut; then chunk c is layers [c * chunk_layers, ...).
    const uint32_t want_planes = 2u * (uint32_t)e->cfg.chunk_layers;
    const bool lay_out = want_planes && no > 0 && po.blocks_per_chunk >= (uint32_t)no &&
                         po.planes_per_chunk == std::min(want_planes, e->n_planes);
    const bool lay_in = want_planes && ni > 0 && pi.blocks_per_chunk >= (uint32_t)ni &&
                        pi.planes_per_chunk == std::min(want_planes, e->n_planes);
    const bool layered = (lay_out || no == 0) && (lay_in || ni == 0);
    e->layer_chunk = layered ? e->cfg.chunk_layers : 0;
    e->layer_on_out = layered && no > 0;
    e->layer_on_in = layered && ni > 0;
    while (!co.done || !ci.done) {
        if (!co.done) {
            const uint32_t j1 = std::min<uint32_t>(co.j0 + po.blocks_per_chunk, (uint32_t)no);
            const uint32_t p1 = std::min<uint32_t>(co.p0 + po.planes_per_chunk, e->n_planes);
            if (cap_wgs > 0) {
                MoveParams p = stage_params(e, e->stage_out, j1 - co.j0, co.p0, p1 - co.p0, U);
                p.out = DirDesc{j1 - co.j0, 0, 1, 0};
                if (!dir_tiles(p.out.n, p.n_planes, p.tiles_per_seg, p.out.tiles)) return KV_EUNSUP;
                launch_move(U, e->vec, (int)std::min<uint32_t>((uint32_t)cap_wgs, p.out.tiles), dkv::kThreads, e->s_out,
                            p, MoveIds{d_out + co.j0, nullptr, nullptr, nullptr}, false);
            } else {
                dkv::StageParams q;
                if (!stage_kernel_params(e, e->stage_out, j1 - co.j0, co.p0, p1 - co.p0, q)) return KV_EUNSUP;
                launch_stage<false>(e->vec, e->s_out, q, d_out + co.j0);
            }
            HIPTRY(e, hipGetLastError());
            if (chunk_copies(e, true, e->stage_out, h_out + no, co.j0, j1, co.p0, p1, e->s_out, n_ops) != KV_OK)
                return KV_EHIP;
            if (layered) HIPTRY(e, hipEventRecord(e->layer_ev_out[co.p0 / po.planes_per_chunk], e->s_out));
            n_ops++;
            co.p0 = p1;
            if (co.p0 >= e->n_planes) { co.p0 = 0; co.j0 = j1; }
            co.done = co.j0 >= (uint32_t)no;
        }
        if (!ci.done) {
            const uint32_t j1 = std::min<uint32_t>(ci.j0 + pi.blocks_per_chunk, (uint32_t)ni);
            const uint32_t p1 = std::min<uint32_t>(ci.p0 + pi.planes_per_chunk, e->n_planes);
            if (chunk_copies(e, false, e->stage_in, h_in + ni, ci.j0, j1, ci.p0, p1, e->s_in, n_ops) != KV_OK)
                return KV_EHIP;
            if (cap_wgs > 0) {
                MoveParams p = stage_params(e, e->stage_in, j1 - ci.j0, ci.p0, p1 - ci.p0, U);
                p.in = DirDesc{j1 - ci.j0, 0, 1, 0};
                if (!dir_tiles(p.in.n, p.n_planes, p.tiles_per_seg, p.in.tiles)) return KV_EUNSUP;
                launch_move(U, e->vec, (int)std::min<uint32_t>((uint32_t)cap_wgs, p.in.tiles), dkv::kThreads, e->s_in, p,
                            MoveIds{nullptr, nullptr, d_in + ci.j0, nullptr}, false);
            } else {
                dkv::StageParams q;
                if (!stage_kernel_params(e, e->stage_in, j1 - ci.j0, ci.p0, p1 - ci.p0, q)) return KV_EUNSUP;
                launch_stage<true>(e->vec, e->s_in, q, d_in + ci.j0);
            }
            HIPTRY(e, hipGetLastError());
            if (layered) HIPTRY(e, hipEventRecord(e->layer_ev_in[ci.p0 / pi.planes_per_chunk], e->s_in));
            n_ops++;
            ci.p0 = p1;
            if (ci.p0 >= e->n_planes) { ci.p0 = 0; ci.j0 = j1; }
            ci.done = ci.j0 >= (uint32_t)ni;
        }
    }
    if (no > 0 && mark_end(e, true, k, e->s_out) != KV_OK) return KV_EHIP;
    if (ni > 0 && mark_end(e, false, k, e->s_in) != KV_OK) return KV_EHIP;
    e->acc.n_launches += n_ops;
    return KV_OK;
}

int ensure_staging(kv_engine *e)
{
    if (e->stage_out) return KV_OK;
    // 256 MiB chunks keep the kernel <-> copy hand-overs (tens of microseconds
    // each) under 1 % of a chunk's link time
    uint64_t cap = e->cfg.staging_bytes ? e->cfg.staging_bytes : (256ull << 20);
    cap -= cap % 256;
    if (cap < 2 * e->seg) return KV_EINVAL;
    e->chunk_cap = cap;
    if (hipMalloc((void **)&e->stage_out, cap) != hipSuccess || hipMalloc((void **)&e->stage_in, cap) != hipSuccess) {
        (void)hipGetLastError();
        return KV_ENOMEM;
    }
    return KV_OK;
}

int transfer(kv_engine *e, const int32_t *oi, const int32_t *os, int32_t no, const int32_t *ii,
             const int32_t *is, int32_t ni)
{
    if (!e) return KV_EINVAL;
    if (e->sticky != KV_OK) return e->sticky;
    int rc = admit(&e->cfg, e->marks, oi, os, no, ii, is, ni);
    if (rc != KV_OK) return rc;
    if (no == 0 && ni == 0) return KV_OK;
    int path = e->cfg.path;
    if (path == KV_PATH_AUTO) path = (no > 0 && ni > 0) ? KV_PATH_FUSED : KV_PATH_ZEROCOPY;
    // The block table orders its own calls across the two streams; for everyone
    // else a call that would race with un-waited work on the other stream is
    // refused.  One launch for both directions joins the streams instead.
    const bool joins = path == KV_PATH_FUSED && no > 0 && ni > 0;
    if (!e->in_after_out && !joins && e->hazards.races(oi, os, no, ii, is, ni)) return KV_EBUSY;
    if (path == KV_PATH_SDMA_STAGED) {
        rc = ensure_staging(e);
        if (rc != KV_OK) return rc;
    }
    open_batch(e);
    e->layer_chunk = 0;  // the kernel paths set it again when they run layer by layer
    if (path == KV_PATH_NAIVE) {
        rc = run_naive(e, oi, os, no, ii, is, ni);
    } else if (path == KV_PATH_DMA_BLOCKS) {
        rc = run_dma_blocks(e, oi, os, no, ii, is, ni);
    } else {
        int k;
        rc = acquire_ring(e, k);
        if (rc != KV_OK) return rc;
        int32_t *dh = e->desc_host + (size_t)k * e->desc_cap;
        if (path != KV_PATH_SDMA_STAGED) {
            int32_t *po = dh, *pi = dh + 2 * (size_t)no;
            if (no) {
                memcpy(po, oi, (size_t)no * sizeof(int32_t));
                memcpy(po + no, os, (size_t)no * sizeof(int32_t));
            }
            if (ni) {
                memcpy(pi, ii, (size_t)ni * sizeof(int32_t));
                memcpy(pi + ni, is, (size_t)ni * sizeof(int32_t));
            }
            rc = run_zero_copy(e, path, k, no, ni);
        } else {
            rc = run_staged(e, k, oi, os, no, ii, is, ni);
        }
    }
    if (rc != KV_OK) return rc;
    if (joins) e->hazards.join();
    else e->hazards.stamp(oi, os, no, ii, is, ni);
    e->acc.bytes_out += (uint64_t)no * e->block_bytes;
    e->acc.bytes_in += (uint64_t)ni * e->block_bytes;
    e->acc.path_used = path;
    return KV_OK;
}

void free_engine(kv_engine *e)
{
    if (!e) return;
    auto ev = [](hipEvent_t &x) { if (x) { (void)hipEventDestroy(x); x = nullptr; } };
    for (int k = 0; k < kRing; k++) { ev(e->ring_out[k]); ev(e->ring_in[k]); }
    ev(e->ev_o0); ev(e->ev_o1); ev(e->ev_i0); ev(e->ev_i1); ev(e->ev_join); ev(e->ev_join_in);
    for (hipEvent_t &x : e->layer_ev_out) ev(x);
    for (hipEvent_t &x : e->layer_ev_in) ev(x);
    if (e->stage_out) (void)hipFree(e->stage_out);
    if (e->stage_in) (void)hipFree(e->stage_in);
    if (e->s_read) (void)hipStreamDestroy(e->s_read);
    if (e->read_ids) (void)hipFree(e->read_ids);
    if (e->read_ids_host) (void)hipHostFree(e->read_ids_host);
    if (e->read_acc) (void)hipFree(e->read_acc);
    if (e->read_acc_host) (void)hipHostFree(e->read_acc_host);
    for (hipEvent_t &x : e->read_ev) ev(x);
    if (e->desc_host) (void)hipHostFree(e->desc_host);
    if (e->desc_dev) (void)hipFree(e->desc_dev);
    if (e->claim) (void)hipFree(e->claim);
    if (e->own_pool && e->pool) (void)hipHostFree(e->pool);
    if (e->own_streams) {
        if (e->s_out) (void)hipStreamDestroy(e->s_out);
        if (e->s_in) (void)hipStreamDestroy(e->s_in);
    }
    delete e;
}

// ---- the entry point that allocates nothing --------------------------------
// Everything kv_rotate keeps in memory the engine allocated (the step counters
// of the move kernel and the device copy of the call's four id lists) lives,
// for kv_rotate_static, in one file-scope array of device memory.  Every GPU the
// library runs on holds its own copy of the array, at its own address, until
// the process ends.  Layout: [0, 256) the counter pair, then the id lists as
// [out_ids | out_slots | in_ids | in_slots].
constexpr size_t kStaticIdsOff = 256;
constexpr size_t kStaticBytes = kStaticIdsOff + 2 * (size_t)KV_STATIC_MAX_BLOCKS * sizeof(int32_t);
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

// In host code `scratch` is only a handle for the symbol, not a device address;
// the address on the current device comes from hipGetSymbolAddress, once per
// device, and only that pointer is ever handed to a kernel.
constexpr int kStaticMaxDevices = 64;
unsigned char *g_scratch_ptr[kStaticMaxDevices] = {};

int static_scratch(unsigned char *&ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kStaticMaxDevices) {
        (void)hipGetLastError();
        return KV_EHIP;
    }
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        const hipError_t err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess || !p) {
            (void)hipGetLastError();
            fprintf(stderr, "duplexkv: hipGetSymbolAddress(scratch) failed on device %d: %s\n", dev,
                    hipGetErrorString(err));
            return KV_EHIP;
        }
        g_scratch_ptr[dev] = (unsigned char *)p;
    }
    ptr = g_scratch_ptr[dev];
    return KV_OK;
}

// The id lists travel to the scratch array as kernel arguments (copied at
// launch, so the caller's arrays are free again when the call returns, and no
// pinned staging buffer is needed): kIdsPerLaunch ints per launch.  The first
// launch of a call also puts the counter pair to zero.
constexpr uint32_t kIdsPerLaunch = 960;
struct IdChunk {
    int32_t v[kIdsPerLaunch];
};

__global__ __launch_bounds__(256) void kv_ids_kernel(const IdChunk c, int32_t *dst, uint32_t n,
                                                     unsigned int *zero)
{
    for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) dst[i] = c.v[i];
    if (zero && threadIdx.x < 2) zero[threadIdx.x] = 0u;
}

// Admission without marks of cache size: sorted copies in static host arrays.
int32_t g_sorted[4][KV_STATIC_MAX_BLOCKS];

bool sorted_has_repeat(const int32_t *p, int32_t n)
{
    for (int32_t i = 1; i < n; i++)
        if (p[i] == p[i - 1]) return true;
    return false;
}

bool sorted_share(const int32_t *a, int32_t na, const int32_t *b, int32_t nb)
{
    int32_t i = 0, j = 0;
    while (i < na && j < nb) {
        if (a[i] == b[j]) return true;
        if (a[i] < b[j]) i++;
        else j++;
    }
    return false;
}

int admit_static(const kv_config *c, const int32_t *oi, const int32_t *os, int32_t no, const int32_t *ii,
                 const int32_t *is, int32_t ni)
{
    if (list_bad(oi, no) || list_bad(os, no) || list_bad(ii, ni) || list_bad(is, ni)) return KV_EINVAL;
    if ((int64_t)no + ni > KV_STATIC_MAX_BLOCKS) return KV_E2BIG;
    if (out_of_range(oi, no, c->n_hbm_blocks) || out_of_range(ii, ni, c->n_hbm_blocks) ||
        out_of_range(os, no, c->n_host_slots) || out_of_range(is, ni, c->n_host_slots))
        return KV_ERANGE;
    const int32_t *src[4] = {oi, os, ii, is};
    const int32_t len[4] = {no, no, ni, ni};
    bool dup = false;
    for (int k = 0; k < 4; k++) {
        if (len[k]) memcpy(g_sorted[k], src[k], (size_t)len[k] * sizeof(int32_t));
        std::sort(g_sorted[k], g_sorted[k] + len[k]);
        dup = dup || sorted_has_repeat(g_sorted[k], len[k]);
    }
    if (dup) return KV_EDUP;
    if (sorted_share(g_sorted[0], no, g_sorted[2], ni) || sorted_share(g_sorted[1], no, g_sorted[3], ni))
        return KV_EOVERLAP;
    return KV_OK;
}

double median(std::vector<double> v)
{
    std::sort(v.begin(), v.end());
    return v[v.size() / 2];
}

}  // namespace

int dkv::drain(kv_engine *e)
{
    if (!e) return KV_EINVAL;
    if (e->sticky != KV_OK) return e->sticky;
    if (e->out_pending) HIPTRY(e, hipStreamSynchronize(e->s_out));
    if (e->in_pending) HIPTRY(e, hipStreamSynchronize(e->s_in));
    e->idle_epoch++;
    return KV_OK;
}

extern "C" {

uint64_t kv_seg_bytes(const kv_config *c) { return config_ok(c) ? seg_of(c) : 0; }
uint64_t kv_block_bytes(const kv_config *c) { return config_ok(c) ? 2ull * c->n_layers * seg_of(c) : 0; }
uint64_t kv_cache_bytes(const kv_config *c)
{
    return config_ok(c) ? kv_block_bytes(c) * (uint64_t)c->n_hbm_blocks : 0;
}
uint64_t kv_pool_bytes(const kv_config *c)
{
    return config_ok(c) ? kv_block_bytes(c) * (uint64_t)c->n_host_slots : 0;
}

int kv_validate(const kv_config *cfg, const int32_t *oi, const int32_t *os, int32_t no, const int32_t *ii,
                const int32_t *is, int32_t ni)
{
    if (!config_ok(cfg)) return KV_EINVAL;
    Marks mk;
    mk.reset((size_t)cfg->n_hbm_blocks, (size_t)cfg->n_host_slots);
    return admit(cfg, mk, oi, os, no, ii, is, ni);
}

int kv_create(kv_engine **out, const kv_config *cfg, void *hbm_cache, void *host_pool, void *stream_out,
              void *stream_in)
{
    if (!out) return KV_EINVAL;
    *out = nullptr;
    if (!config_ok(cfg) || !hbm_cache) return KV_EINVAL;
    if ((stream_out == nullptr) != (stream_in == nullptr)) return KV_EINVAL;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) {
        (void)hipGetLastError();
        fprintf(stderr, "duplexkv: no HIP device is visible\n");
        return KV_EHIP;
    }
    kv_engine *e = new (std::nothrow) kv_engine;
    if (!e) return KV_ENOMEM;
    e->cfg = *cfg;
    e->seg = seg_of(cfg);
    e->n_planes = 2u * (uint32_t)cfg->n_layers;
    e->block_bytes = kv_block_bytes(cfg);
    e->cache_bytes = kv_cache_bytes(cfg);
    e->pool_bytes = kv_pool_bytes(cfg);
    e->hbm = (uint8_t *)hbm_cache;
    int rc = KV_OK;
    auto fail = [&](int code) { free_engine(e); return code; };

    if (hipGetDevice(&e->device) != hipSuccess) return fail(KV_EHIP);
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, e->device) != hipSuccess) return fail(KV_EHIP);
    e->n_cus = prop.multiProcessorCount;

    // the cache pointer must be a device allocation that really spans cache_bytes
    {
        hipDeviceptr_t base = nullptr;
        size_t span = 0;
        if (hipMemGetAddressRange(&base, &span, (hipDeviceptr_t)hbm_cache) != hipSuccess) {
            (void)hipGetLastError();
            fprintf(stderr, "duplexkv: hbm_cache is not a device allocation\n");
            return fail(KV_EINVAL);
        }
        const uintptr_t lo = (uintptr_t)base, hi = lo + span, p = (uintptr_t)hbm_cache;
        if (p < lo || p + e->cache_bytes > hi) {
            fprintf(stderr, "duplexkv: hbm_cache allocation is smaller than the configured cache\n");
            return fail(KV_EINVAL);
        }
    }
    if (host_pool) {
        hipPointerAttribute_t at;
        if (hipPointerGetAttributes(&at, host_pool) != hipSuccess || at.type != hipMemoryTypeHost) {
            (void)hipGetLastError();
            fprintf(stderr, "duplexkv: host_pool is not pinned host memory\n");
            return fail(KV_EINVAL);
        }
        hipDeviceptr_t base = nullptr;
        size_t span = 0;
        if (hipMemGetAddressRange(&base, &span, (hipDeviceptr_t)host_pool) == hipSuccess) {
            const uintptr_t lo = (uintptr_t)base, hi = lo + span, p = (uintptr_t)host_pool;
            if (p < lo || p + e->pool_bytes > hi) {
                fprintf(stderr, "duplexkv: host_pool allocation is smaller than the configured pool\n");
                return fail(KV_EINVAL);
            }
        } else {
            (void)hipGetLastError();
        }
        e->pool = (uint8_t *)host_pool;
    } else {
        if (hipHostMalloc((void **)&e->pool, e->pool_bytes, hipHostMallocDefault) != hipSuccess) {
            (void)hipGetLastError();
            e->pool = nullptr;
            return fail(KV_ENOMEM);
        }
        e->own_pool = true;
    }
    e->vec = pick_vec(e);

    if (stream_out) {
        e->s_out = (hipStream_t)stream_out;
        e->s_in = (hipStream_t)stream_in;
    } else {
        e->own_streams = true;
        if (hipStreamCreateWithFlags(&e->s_out, hipStreamNonBlocking) != hipSuccess ||
            hipStreamCreateWithFlags(&e->s_in, hipStreamNonBlocking) != hipSuccess)
            return fail(KV_EHIP);
    }
    // one call names at most min(blocks, slots) ids over both directions
    e->desc_cap = 2 * (size_t)std::min(cfg->n_hbm_blocks, cfg->n_host_slots) + 16;
    if (hipHostMalloc((void **)&e->desc_host, kRing * e->desc_cap * sizeof(int32_t), hipHostMallocDefault) !=
            hipSuccess ||
        hipMalloc((void **)&e->desc_dev, kRing * e->desc_cap * sizeof(int32_t)) != hipSuccess ||
        hipMalloc((void **)&e->claim, 2 * kClaimStride * sizeof(unsigned int)) != hipSuccess) {
        (void)hipGetLastError();
        return fail(KV_ENOMEM);
    }
    // the tile counters start at zero; every launch leaves them at zero again
    if (hipMemset(e->claim, 0, 2 * kClaimStride * sizeof(unsigned int)) != hipSuccess)
        return fail(KV_EHIP);
    bool ok = true;
    for (int k = 0; k < kRing; k++) {
        ok = ok && hipEventCreate(&e->ring_out[k]) == hipSuccess;
        ok = ok && hipEventCreate(&e->ring_in[k]) == hipSuccess;
    }
    for (hipEvent_t *x : {&e->ev_o0, &e->ev_o1, &e->ev_i0, &e->ev_i1}) ok = ok && hipEventCreate(x) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&e->ev_join, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&e->ev_join_in, hipEventDisableTiming) == hipSuccess;
    if (cfg->chunk_layers > 0) {
        e->layer_n_chunks = (cfg->n_layers + cfg->chunk_layers - 1) / cfg->chunk_layers;
        e->layer_ev_out.assign((size_t)e->layer_n_chunks, nullptr);
        e->layer_ev_in.assign((size_t)e->layer_n_chunks, nullptr);
        for (hipEvent_t &x : e->layer_ev_out) ok = ok && hipEventCreateWithFlags(&x, hipEventDisableTiming) == hipSuccess;
        for (hipEvent_t &x : e->layer_ev_in) ok = ok && hipEventCreateWithFlags(&x, hipEventDisableTiming) == hipSuccess;
    }
    if (!ok) return fail(KV_EHIP);
    e->marks.reset((size_t)cfg->n_hbm_blocks, (size_t)cfg->n_host_slots);
    e->hazards.reset((size_t)cfg->n_hbm_blocks, (size_t)cfg->n_host_slots);
    if (cfg->path == KV_PATH_SDMA_STAGED) {
        rc = ensure_staging(e);
        if (rc != KV_OK) return fail(rc);
    }
    *out = e;
    return KV_OK;
}

int kv_destroy(kv_engine *e)
{
    if (!e) return KV_EINVAL;
    if (e->n_tables > 0) return KV_EBUSY;  // a block table still points at this engine
    if (e->s_read) (void)hipStreamSynchronize(e->s_read);
    (void)hipStreamSynchronize(e->s_out);
    (void)hipStreamSynchronize(e->s_in);
    free_engine(e);
    return KV_OK;
}

int kv_swap_out(kv_engine *e, const int32_t *ids, const int32_t *slots, int32_t n)
{
    return transfer(e, ids, slots, n, nullptr, nullptr, 0);
}

int kv_swap_in(kv_engine *e, const int32_t *slots, const int32_t *ids, int32_t n)
{
    return transfer(e, nullptr, nullptr, 0, ids, slots, n);
}

int kv_rotate(kv_engine *e, const int32_t *oi, const int32_t *os, int32_t no, const int32_t *ii,
              const int32_t *is, int32_t ni)
{
    return transfer(e, oi, os, no, ii, is, ni);
}

int kv_wait(kv_engine *e)
{
    if (!e) return KV_EINVAL;
    if (e->sticky != KV_OK) return e->sticky;
    // Only streams this engine put work on are waited for.
    for (int side = 0; side < 2; side++) {
        const bool pending = side == 0 ? e->out_pending : e->in_pending;
        if (!pending) continue;
        HIPTRY(e, hipStreamSynchronize(side == 0 ? e->s_out : e->s_in));
    }
    e->out_pending = e->in_pending = false;
    e->out_dirty = e->in_dirty = false;
    e->hazards.join();
    e->idle_epoch++;
    for (int k = 0; k < kRing; k++) e->ring_out_rec[k] = e->ring_in_rec[k] = false;
    if (e->batch_open) {
        e->acc.ms_e2e = now_ms() - e->t0;
        float ms = 0;
        if (e->b_o0 && e->b_o1) {
            HIPTRY(e, hipEventElapsedTime(&ms, e->b_o0, e->b_o1));
            e->acc.ms_out = ms;
        }
        if (e->b_i0 && e->b_i1) {
            HIPTRY(e, hipEventElapsedTime(&ms, e->b_i0, e->b_i1));
            e->acc.ms_in = ms;
        }
        e->last = e->acc;
        e->batch_open = false;
    }
    return KV_OK;
}

int kv_query(kv_engine *e)
{
    if (!e) return KV_EINVAL;
    if (e->sticky != KV_OK) return e->sticky;
    for (int side = 0; side < 2; side++) {
        const bool pending = side == 0 ? e->out_pending : e->in_pending;
        if (!pending) continue;
        const hipError_t q = hipStreamQuery(side == 0 ? e->s_out : e->s_in);
        if (q == hipErrorNotReady) {
            (void)hipGetLastError();  // not an error: forget it
            return KV_EBUSY;
        }
        HIPTRY(e, q);
    }
    // nothing runs any more, so nothing can race with what comes next
    e->out_dirty = e->in_dirty = false;
    e->hazards.join();
    e->idle_epoch++;
    return KV_OK;
}

// The events behind which `layer` of the most recent transfer call is complete:
// its chunk's events if that call ran layer by layer, else the call's end events.
static int layer_events(kv_engine *e, int32_t layer, hipEvent_t (&out)[2])
{
    out[0] = out[1] = nullptr;
    if (!e || layer < 0 || layer >= e->cfg.n_layers) return KV_EINVAL;
    if (e->sticky != KV_OK) return e->sticky;
    if (e->layer_chunk > 0) {
        const size_t c = (size_t)(layer / e->layer_chunk);
        if (e->layer_on_out) out[0] = e->layer_ev_out[c];
        if (e->layer_on_in) out[1] = e->layer_ev_in[c];
    } else {
        if (e->out_pending) out[0] = e->b_o1;
        if (e->in_pending) out[1] = e->b_i1;
    }
    return KV_OK;
}

int kv_stream_wait_layer(kv_engine *e, void *stream, int32_t layer)
{
    hipEvent_t evs[2];
    const int rc = layer_events(e, layer, evs);
    if (rc != KV_OK) return rc;
    for (hipEvent_t x : evs)
        if (x) HIPTRY(e, hipStreamWaitEvent((hipStream_t)stream, x, 0));
    return KV_OK;
}

int kv_wait_layer(kv_engine *e, int32_t layer)
{
    hipEvent_t evs[2];
    const int rc = layer_events(e, layer, evs);
    if (rc != KV_OK) return rc;
    for (hipEvent_t x : evs)
        if (x) HIPTRY(e, hipEventSynchronize(x));
    return KV_OK;
}

int kv_host_pool(kv_engine *e, void **ptr, uint64_t *bytes)
{
    if (!e || !ptr || !bytes) return KV_EINVAL;
    *ptr = e->pool;
    *bytes = e->pool_bytes;
    return KV_OK;
}

int kv_last_stats(kv_engine *e, kv_stats *out)
{
    if (!e || !out) return KV_EINVAL;
    *out = e->last;
    return KV_OK;
}

int kv_rotate_static(const kv_config *cfg, void *hbm_cache, void *host_pool, void *stream,
                     const int32_t *oi, const int32_t *os, int32_t no, const int32_t *ii, const int32_t *is,
                     int32_t ni)
{
    if (!config_ok(cfg) || !hbm_cache || !host_pool) return KV_EINVAL;
    if (cfg->path != KV_PATH_AUTO && cfg->path != KV_PATH_FUSED) return KV_EUNSUP;
    // the host-side arrays (sorted copies, the argument chunk, the address table) are the
    // process's, not the call's: callers on several threads take turns
    static std::mutex turn;
    std::lock_guard<std::mutex> hold(turn);
    int rc = admit_static(cfg, oi, os, no, ii, is, ni);
    if (rc != KV_OK) return rc;
    // an engine that exists only on this stack frame, so that the launch helpers
    // of the other paths serve here too; nothing in it owns memory
    kv_engine view;
    kv_engine *e = &view;
    e->cfg = *cfg;
    e->seg = seg_of(cfg);
    e->n_planes = 2u * (uint32_t)cfg->n_layers;
    e->block_bytes = kv_block_bytes(cfg);
    e->cache_bytes = kv_cache_bytes(cfg);
    e->pool_bytes = kv_pool_bytes(cfg);
    e->hbm = (uint8_t *)hbm_cache;
    e->pool = (uint8_t *)host_pool;
    e->vec = pick_vec(e);
    // both pointers are checked before a kernel is given them
    {
        hipDeviceptr_t base = nullptr;
        size_t span = 0;
        if (hipMemGetAddressRange(&base, &span, (hipDeviceptr_t)hbm_cache) != hipSuccess ||
            (uintptr_t)hbm_cache + e->cache_bytes > (uintptr_t)base + span) {
            (void)hipGetLastError();
            fprintf(stderr, "duplexkv: hbm_cache is not a device allocation of the configured size\n");
            return KV_EINVAL;
        }
        hipPointerAttribute_t at;
        if (hipPointerGetAttributes(&at, host_pool) != hipSuccess || at.type != hipMemoryTypeHost) {
            (void)hipGetLastError();
            fprintf(stderr, "duplexkv: host_pool is not pinned host memory\n");
            return KV_EINVAL;
        }
        if (hipMemGetAddressRange(&base, &span, (hipDeviceptr_t)host_pool) == hipSuccess) {
            if ((uintptr_t)host_pool + e->pool_bytes > (uintptr_t)base + span) {
                fprintf(stderr, "duplexkv: host_pool allocation is smaller than the configured pool\n");
                return KV_EINVAL;
            }
        } else {
            (void)hipGetLastError();
        }
    }
    if (no == 0 && ni == 0) return KV_OK;
    const LinkKind kind = no == 0 ? kInOnly : ni == 0 ? kOutOnly : ni >= 2 * (int64_t)no ? kInHeavy : kBoth;
    const LinkShape sh = link_shape(e, kind);
    MoveParams p = base_params(e, sh.u);
    p.far_out = p.far_in = e->pool;
    pool_strides(e, p.far_slot_stride_out, p.far_plane_stride_out);
    p.far_slot_stride_in = p.far_slot_stride_out;
    p.far_plane_stride_in = p.far_plane_stride_out;
    p.plane_major = cfg->host_layout == KV_HOST_LAYER_FIRST ? 1u : 0u;
    p.out = DirDesc{(uint32_t)no, 0, 0, 0};
    p.in = DirDesc{(uint32_t)ni, 0, 0, 0};
    if (!dir_tiles(p.out.n, p.n_planes, p.tiles_per_seg, p.out.tiles) ||
        !dir_tiles(p.in.n, p.n_planes, p.tiles_per_seg, p.in.tiles))
        return KV_EUNSUP;
    if (p.out.tiles > 0 && p.in.tiles > p.out.tiles)
        p.mix_q = (((uint64_t)p.out.tiles << 32) + p.in.tiles - 1) / p.in.tiles;
    unsigned char *sc = nullptr;
    rc = static_scratch(sc);
    if (rc != KV_OK) return rc;
    p.claim = reinterpret_cast<unsigned int *>(sc);
    int32_t *ids = reinterpret_cast<int32_t *>(sc + kStaticIdsOff);
    hipStream_t s = (hipStream_t)stream;
    // the four lists, back to back, through kernel arguments
    const int32_t *src[4] = {oi, os, ii, is};
    const uint32_t len[4] = {(uint32_t)no, (uint32_t)no, (uint32_t)ni, (uint32_t)ni};
    const uint32_t total = 2u * ((uint32_t)no + (uint32_t)ni);
    static IdChunk chunk;  // one caller at a time
    uint32_t done = 0, list = 0, at = 0;
    while (done < total) {
        uint32_t n = 0;
        while (n < kIdsPerLaunch && list < 4) {
            const uint32_t take = std::min(kIdsPerLaunch - n, len[list] - at);
            if (take) memcpy(chunk.v + n, src[list] + at, (size_t)take * sizeof(int32_t));
            n += take;
            at += take;
            if (at == len[list]) { list++; at = 0; }
        }
        hipLaunchKernelGGL(kv_ids_kernel, dim3(1), dim3(256), 0, s, chunk, ids + done, n,
                           done == 0 ? p.claim : (unsigned int *)nullptr);
        HIPTRY((kv_engine *)nullptr, hipGetLastError());
        done += n;
    }
    launch_move(sh.u, e->vec, sh.wgs, sh.lanes, s, p,
                MoveIds{ids, ids + no, ids + 2 * (size_t)no, ids + 2 * (size_t)no + ni}, true);
    HIPTRY((kv_engine *)nullptr, hipGetLastError());
    return KV_OK;
}

int kv_probe_link(uint64_t bytes, int32_t reps, double *d2h, double *h2d, double *d2h_duplex,
                  double *h2d_duplex)
{
    if (bytes == 0 || reps <= 0 || !d2h || !h2d || !d2h_duplex || !h2d_duplex) return KV_EINVAL;
    kv_engine *e = nullptr;  // HIPTRY wants one; no engine state here
    void *ha = nullptr, *hb = nullptr, *da = nullptr, *db = nullptr;
    // Streams share a few hardware queues and DMA engines; which pair a process
    // gets depends on what else it has created.  Up to three rounds of five
    // streams each (more than the process has hardware queues; earlier rounds'
    // streams stay alive so that later ones land elsewhere): every pairing with
    // a round's first two streams is timed and the best one is reported, the
    // link's ceiling and not a property of one unlucky pairing.  A round that
    // already shows the directions overlapping ends the search.
    constexpr int kS = 5, kRounds = 3;
    hipStream_t st[kS * kRounds] = {};
    auto cleanup = [&]() {
        if (ha) (void)hipHostFree(ha);
        if (hb) (void)hipHostFree(hb);
        if (da) (void)hipFree(da);
        if (db) (void)hipFree(db);
        for (int i = 0; i < kS * kRounds; i++)
            if (st[i]) (void)hipStreamDestroy(st[i]);
    };
    if (hipHostMalloc(&ha, bytes, hipHostMallocDefault) != hipSuccess ||
        hipHostMalloc(&hb, bytes, hipHostMallocDefault) != hipSuccess ||
        hipMalloc(&da, bytes) != hipSuccess || hipMalloc(&db, bytes) != hipSuccess) {
        (void)hipGetLastError();
        cleanup();
        return KV_ENOMEM;
    }
    memset(ha, 1, bytes);
    memset(hb, 2, bytes);
    // one timed pass: D2H on `so` and / or H2D on `si`; returns wall ms to the last completion
    auto pass = [&](hipStream_t so, hipStream_t si, double &ms) -> int {
        std::vector<double> t;
        for (int it = 0; it < reps + 2; it++) {
            HIPTRY(e, hipDeviceSynchronize());
            const double a = now_ms();
            if (so) HIPTRY(e, hipMemcpyAsync(ha, da, bytes, hipMemcpyDeviceToHost, so));
            if (si) HIPTRY(e, hipMemcpyAsync(db, hb, bytes, hipMemcpyHostToDevice, si));
            if (so) HIPTRY(e, hipStreamSynchronize(so));
            if (si) HIPTRY(e, hipStreamSynchronize(si));
            if (it >= 2) t.push_back(now_ms() - a);
        }
        ms = median(t);
        return KV_OK;
    };
    auto body = [&]() -> int {
        HIPTRY(e, hipMemset(da, 3, bytes));
        HIPTRY(e, hipMemset(db, 4, bytes));
        double ms = 0, best = 1e30, one_way = 0;
        const int pairs[7][2] = {{0, 1}, {0, 2}, {0, 3}, {0, 4}, {1, 2}, {1, 3}, {1, 4}};
        for (int r = 0; r < kRounds; r++) {
            hipStream_t *q = st + r * kS;
            for (int i = 0; i < kS; i++) HIPTRY(e, hipStreamCreateWithFlags(&q[i], hipStreamNonBlocking));
            if (r == 0) {
                if (pass(q[0], nullptr, ms) != KV_OK) return KV_EHIP;
                *d2h = bytes / ms / 1e6;
                one_way = ms;
                if (pass(nullptr, q[1], ms) != KV_OK) return KV_EHIP;
                *h2d = bytes / ms / 1e6;
                one_way = std::max(one_way, ms);
            }
            for (auto &pr : pairs) {
                if (pass(q[pr[0]], q[pr[1]], ms) != KV_OK) return KV_EHIP;
                best = std::min(best, ms);
            }
            if (best < 1.5 * one_way) break;  // the two copies overlapped
        }
        // both directions are charged the wall time of the pair
        *d2h_duplex = *h2d_duplex = bytes / best / 1e6;
        return KV_OK;
    };
    int rc = body();
    (void)hipDeviceSynchronize();
    cleanup();
    return rc;
}

int kv_reader_start(kv_engine *e, const int32_t *ids, int32_t n, int32_t passes, int32_t max_wgs)
{
    if (!e || list_bad(ids, n) || passes < 1 || passes > 256 || max_wgs < 0) return KV_EINVAL;
    if (e->sticky != KV_OK) return e->sticky;
    if (e->read_passes != 0) return KV_EINVAL;  // previous reader not waited for
    if (out_of_range(ids, n, e->cfg.n_hbm_blocks)) return KV_ERANGE;
    if ((int64_t)n > 2 * (int64_t)e->cfg.n_hbm_blocks) return KV_EINVAL;
    if (e->seg % 16 != 0 || ((uintptr_t)e->hbm & 15u) != 0) return KV_EUNSUP;
    if (!e->s_read) {
        const size_t idb = 2 * (size_t)e->cfg.n_hbm_blocks * sizeof(int32_t);
        if (hipMalloc((void **)&e->read_ids, idb) != hipSuccess ||
            hipHostMalloc((void **)&e->read_ids_host, idb, hipHostMallocDefault) != hipSuccess ||
            hipMalloc((void **)&e->read_acc, sizeof(unsigned long long) + 256 * sizeof(unsigned int)) != hipSuccess ||
            hipHostMalloc((void **)&e->read_acc_host, sizeof(unsigned long long), hipHostMallocDefault) !=
                hipSuccess) {
            (void)hipGetLastError();
            return KV_ENOMEM;
        }
        HIPTRY(e, hipStreamCreateWithFlags(&e->s_read, hipStreamNonBlocking));
    }
    while ((int32_t)e->read_ev.size() < passes + 1) {
        hipEvent_t x;
        HIPTRY(e, hipEventCreate(&x));
        e->read_ev.push_back(x);
    }
    constexpr int U = 8;
    dkv::ReadParams p{};
    p.hbm = e->hbm;
    p.ids = e->read_ids;
    p.acc = e->read_acc;
    hbm_strides(e, p.hbm_plane_stride, p.hbm_block_stride);
    p.n = (uint32_t)n;
    p.n_planes = e->n_planes;
    p.vec_per_seg = (uint32_t)(e->seg / 16);
    p.tiles_per_seg = (p.vec_per_seg + dkv::kThreads * U - 1) / (dkv::kThreads * U);
    if (!dir_tiles(p.n, p.n_planes, p.tiles_per_seg, p.tiles)) return KV_EUNSUP;
    *e->read_acc_host = 0;
    HIPTRY(e, hipMemsetAsync(e->read_acc, 0, sizeof(unsigned long long) + 256 * sizeof(unsigned int), e->s_read));
    if (n > 0) {
        memcpy(e->read_ids_host, ids, (size_t)n * sizeof(int32_t));
        HIPTRY(e, hipMemcpyAsync(e->read_ids, e->read_ids_host, (size_t)n * sizeof(int32_t),
                                 hipMemcpyHostToDevice, e->s_read));
    }
    // Measured per pass over 37.5 GiB, TB/s by workgroups per CU (claims of 32
    // tiles): 4 -> 5.70, 5 -> 6.56, 5.5 -> 6.68, 6 -> 6.75, 8 -> 6.85.  From 6 per
    // CU on the persistent workgroups hold so much of every CU for a whole pass
    // (~6 ms) that another kernel's waves wait for the pass to end before they
    // start, which no model execution made of many short kernels would do to a
    // rotation; 5.5 per CU gives up 2 % and leaves that room.
    int wgs = 11 * (e->n_cus > 0 ? e->n_cus : 256) / 2;
    if (max_wgs > 0) wgs = std::min(wgs, (int)max_wgs);
    wgs = (int)std::min<uint32_t>((uint32_t)wgs, std::max<uint32_t>(p.tiles, 1u));
    HIPTRY(e, hipEventRecord(e->read_ev[0], e->s_read));
    for (int32_t k = 0; k < passes; k++) {
        if (p.tiles > 0) {
            p.next = reinterpret_cast<unsigned int *>(e->read_acc + 1) + k;
            hipLaunchKernelGGL((dkv::kv_reader_kernel<U>), dim3((unsigned)wgs), dim3(dkv::kThreads), 0, e->s_read, p);
            HIPTRY(e, hipGetLastError());
        }
        HIPTRY(e, hipEventRecord(e->read_ev[(size_t)k + 1], e->s_read));
    }
    HIPTRY(e, hipMemcpyAsync(e->read_acc_host, e->read_acc, sizeof(unsigned long long), hipMemcpyDeviceToHost,
                             e->s_read));
    e->read_passes = passes;
    return KV_OK;
}

int kv_reader_wait(kv_engine *e, uint64_t *checksum, double *ms_per_pass)
{
    if (!e || !checksum) return KV_EINVAL;
    if (e->sticky != KV_OK) return e->sticky;
    if (e->read_passes == 0) return KV_EINVAL;
    HIPTRY(e, hipStreamSynchronize(e->s_read));
    *checksum = (uint64_t)*e->read_acc_host;
    if (ms_per_pass) {
        for (int32_t k = 0; k < e->read_passes; k++) {
            float ms = 0;
            HIPTRY(e, hipEventElapsedTime(&ms, e->read_ev[(size_t)k], e->read_ev[(size_t)k + 1]));
            ms_per_pass[k] = ms;
        }
    }
    e->read_passes = 0;
    return KV_OK;
}

const char *kv_strerror(int code)
{
    switch (code) {
    case KV_OK: return "ok";
    case KV_EINVAL: return "invalid argument or configuration";
    case KV_ERANGE: return "block id or host slot out of range";
    case KV_EDUP: return "duplicate id within one list";
    case KV_EOVERLAP: return "block or slot named for both directions";
    case KV_ENOMEM: return "allocation failed";
    case KV_EHIP: return "HIP runtime failure";
    case KV_EUNSUP: return "path cannot serve this shape or request";
    case KV_EBUSY: return "block or slot still in use by an un-waited call on the other stream";
    case KV_ENOSPC: return "not enough free HBM blocks or host slots";
    case KV_E2BIG: return "more blocks than the allocation-free entry point's scratch array holds";
    default: return "unknown code";
    }
}

}  // extern "C"
