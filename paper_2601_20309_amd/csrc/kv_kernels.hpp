// Device kernels of the KV rotation engine (gfx950, wave64).
//
// Everything here is data movement: no MFMA, no arithmetic beyond addressing.
// One kernel family, kv_move_kernel, serves every use:
//   - duplex rotation in ONE launch: each thread alternates a 16-byte move
//     HBM->host with a 16-byte move host->HBM, which keeps the two PCIe
//     directions locked 1:1 (measured faster in duplex than two independent
//     kernels, and equal to the DMA engines' duplex rate);
//   - a single direction (the other list empty): zero-copy swap-out or swap-in;
//   - pack / unpack between the scattered cache and a contiguous staging
//     buffer in HBM (the "far" side is then device memory, slot = list index).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dkv {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;      // default lanes per workgroup (4 waves)
constexpr int kMaxThreads = 1024;  // the move kernels take their tile width from blockDim.x, up to this

// One direction's block list as the kernel sees it.  The id arrays themselves
// are separate __restrict__ kernel arguments so that the compiler fetches them
// with scalar loads (their own counter, off the vector-memory critical path).
struct DirDesc {
    uint32_t n;      // blocks
    uint32_t tiles;  // n * n_planes * tiles_per_seg
    uint32_t iota;   // 1: far-side slot of list entry i is i itself (staging); 0: slots[i]
    uint32_t pad;
};

// Addressing (Section 4.3.1 of the paper: layer x block x segment):
//   HBM  segment (plane, id)   at hbm + plane * hbm_plane_stride + id * hbm_block_stride
//   far  segment (plane, slot) at far + slot * far_slot_stride + plane * far_plane_stride
// `plane` = layer * 2 + (0 for K, 1 for V).
struct MoveParams {
    uint8_t *hbm;
    uint8_t *far_out;  // destination of the out direction (host pool or staging)
    uint8_t *far_in;   // source of the in direction
    uint64_t seg_bytes;
    uint64_t hbm_plane_stride;  // layer-first cache: blocks * seg; block-first cache: seg
    uint64_t hbm_block_stride;  // layer-first cache: seg;          block-first cache: planes * seg
    uint64_t far_slot_stride_out, far_plane_stride_out;
    uint64_t far_slot_stride_in, far_plane_stride_in;
    uint32_t plane0;         // first plane this launch covers
    uint32_t n_planes;       // planes this launch covers
    uint32_t vec_per_seg;    // seg_bytes / sizeof(V)
    uint32_t tiles_per_seg;  // ceil(vec_per_seg / (lanes per workgroup * U))
    uint32_t plane_major;    // tile order: 1 = [plane][i][tile], 0 = [i][plane][tile]
    uint32_t full_tiles;     // 1: vec_per_seg is a multiple of the tile, no lane is ever out of range
    // 0, or ceil(out.tiles * 2^32 / in.tiles) when the in list is the longer one and
    // the out tiles are to be spread evenly over it (see run_in_heavy)
    uint64_t mix_q;
    DirDesc out, in;
};

// Tile t of direction d -> byte offsets (segment base + tile start) on both sides.
__device__ __forceinline__ void locate(const MoveParams &p, const DirDesc &d,
                                       const int32_t *__restrict__ ids,
                                       const int32_t *__restrict__ slots, uint32_t t,
                                       uint64_t slot_stride, uint64_t plane_stride,
                                       uint32_t tile_bytes, uint64_t &hbm_off, uint64_t &far_off)
{
    const uint32_t segidx = t / p.tiles_per_seg;
    const uint32_t tin = t - segidx * p.tiles_per_seg;
    uint32_t i, pl;
    if (p.plane_major) {
        pl = segidx / d.n;
        i = segidx - pl * d.n;
    } else {
        i = segidx / p.n_planes;
        pl = segidx - i * p.n_planes;
    }
    pl += p.plane0;
    const uint32_t id = (uint32_t)ids[i];
    const uint32_t slot = d.iota ? i : (uint32_t)slots[i];
    hbm_off = (uint64_t)pl * p.hbm_plane_stride + (uint64_t)id * p.hbm_block_stride + (uint64_t)tin * tile_bytes;
    far_off = (uint64_t)slot * slot_stride + (uint64_t)pl * plane_stride + (uint64_t)tin * tile_bytes;
}

// Everything one lane needs to move its share of one tile.  Which directions
// take part is a compile-time property of the loop the tile belongs to, so the
// hot loops are straight-line code and the compiler can count exactly how many
// loads may stay in flight at each store.
template <typename V>
struct LaneTile {
    const V *src_i;
    V *dst_i;
    const V *src_o;
    V *dst_o;
};

template <typename V, bool IN, bool OUT>
__device__ __forceinline__ LaneTile<V> lane_tile(const MoveParams &p, const int32_t *__restrict__ out_ids,
                                                 const int32_t *__restrict__ out_slots,
                                                 const int32_t *__restrict__ in_ids,
                                                 const int32_t *__restrict__ in_slots, uint32_t t,
                                                 uint32_t tile_vecs, uint32_t tid)
{
    LaneTile<V> r{nullptr, nullptr, nullptr, nullptr};
    const uint32_t tile_bytes = tile_vecs * (uint32_t)sizeof(V);
    if constexpr (IN) {
        uint64_t ho, fo;
        locate(p, p.in, in_ids, in_slots, t, p.far_slot_stride_in, p.far_plane_stride_in, tile_bytes, ho, fo);
        r.src_i = reinterpret_cast<const V *>(p.far_in + fo) + tid;
        r.dst_i = reinterpret_cast<V *>(p.hbm + ho) + tid;
    }
    if constexpr (OUT) {
        uint64_t ho, fo;
        locate(p, p.out, out_ids, out_slots, t, p.far_slot_stride_out, p.far_plane_stride_out, tile_bytes, ho, fo);
        r.src_o = reinterpret_cast<const V *>(p.hbm + ho) + tid;
        r.dst_o = reinterpret_cast<V *>(p.far_out + fo) + tid;
    }
    return r;
}

// Loads of one full tile: the far-side (host) loads first, they have the long
// latency; then the HBM loads.  No lane predicate: all issue back to back.
template <typename V, int U, bool IN, bool OUT>
__device__ __forceinline__ void tile_loads(const LaneTile<V> &a, uint32_t lanes, V (&vi)[U], V (&vo)[U])
{
    if constexpr (IN) {
#pragma unroll
        for (int u = 0; u < U; u++) vi[u] = a.src_i[u * lanes];
    }
    if constexpr (OUT) {
#pragma unroll
        for (int u = 0; u < U; u++) vo[u] = a.src_o[u * lanes];
    }
}

template <typename V, int U, bool IN, bool OUT>
__device__ __forceinline__ void tile_stores(const LaneTile<V> &a, uint32_t lanes, const V (&vi)[U], const V (&vo)[U])
{
    if constexpr (OUT) {
#pragma unroll
        for (int u = 0; u < U; u++) a.dst_o[u * lanes] = vo[u];
    }
    if constexpr (IN) {
#pragma unroll
        for (int u = 0; u < U; u++) a.dst_i[u * lanes] = vi[u];
    }
}

// Tiles t, t + stride, ... below t_end, all full, all with the same directions.
// Software pipelined in registers: the loads of the workgroup's next tile are
// issued before the stores of the current one, so each lane keeps up to 2 * U
// vectors per direction in flight and the link sees no gap between a
// workgroup's tiles.  Returns the first tile index >= t_end of this workgroup.
template <typename V, int U, bool IN, bool OUT>
__device__ __forceinline__ uint32_t run_full(const MoveParams &p, const int32_t *__restrict__ out_ids,
                                             const int32_t *__restrict__ out_slots,
                                             const int32_t *__restrict__ in_ids,
                                             const int32_t *__restrict__ in_slots, uint32_t t, uint32_t t_end,
                                             uint32_t stride, uint32_t lanes, uint32_t tid)
{
    if (t >= t_end) return t;
    const uint32_t tile_vecs = lanes * U;
    LaneTile<V> cur = lane_tile<V, IN, OUT>(p, out_ids, out_slots, in_ids, in_slots, t, tile_vecs, tid);
    V ai[U], ao[U];
    tile_loads<V, U, IN, OUT>(cur, lanes, ai, ao);
    for (t += stride; t < t_end; t += stride) {
        const LaneTile<V> nxt = lane_tile<V, IN, OUT>(p, out_ids, out_slots, in_ids, in_slots, t, tile_vecs, tid);
        V bi[U], bo[U];
        tile_loads<V, U, IN, OUT>(nxt, lanes, bi, bo);
        tile_stores<V, U, IN, OUT>(cur, lanes, ai, ao);
        cur = nxt;
#pragma unroll
        for (int u = 0; u < U; u++) {
            if constexpr (IN) ai[u] = bi[u];
            if constexpr (OUT) ao[u] = bo[u];
        }
    }
    tile_stores<V, U, IN, OUT>(cur, lanes, ai, ao);
    return t;
}

// The in list is the longer one: its tiles t, t + stride, ... set the pace and
// the out tiles are spread evenly over them, out tile s riding with the in tile
// t at which floor(t * q / 2^32) steps from s to s + 1 (q = ceil(S * 2^32 / L),
// so the steps are 0 or 1 and all S out tiles are met exactly once over the L
// in tiles).  Measured on PCIe Gen5 x16: host->HBM reads can stay at the link's
// one-way rate (55-57 GB/s) while up to ~0.85 as many bytes go the other way
// (47 GB/s), 102 GB/s in all, whereas pairing the lists 1:1 and moving the rest
// of the in list afterwards holds both at 49.5 GB/s for the paired part.  (The
// mirror case gains nothing: with the out list longer, what limits is the
// upstream direction, which carries the out data and the read requests of the
// in data, and that sum does not depend on the order.)  Whether a tile has an
// out tile riding along is uniform over the workgroup.
template <typename V, int U>
__device__ __forceinline__ void run_in_heavy(const MoveParams &p, const int32_t *__restrict__ out_ids,
                                             const int32_t *__restrict__ out_slots,
                                             const int32_t *__restrict__ in_ids,
                                             const int32_t *__restrict__ in_slots, uint32_t t, uint32_t stride,
                                             uint32_t lanes, uint32_t tid)
{
    const uint32_t tile_vecs = lanes * U, n_in = p.in.tiles, n_out = p.out.tiles;
    for (; t < n_in; t += stride) {
        const uint64_t a = (uint64_t)t * p.mix_q, b = a + p.mix_q;
        const uint32_t s0 = (uint32_t)(a >> 32);
        uint32_t s1 = (uint32_t)(b >> 32);
        s1 = s1 < n_out ? s1 : n_out;
        const LaneTile<V> li = lane_tile<V, true, false>(p, out_ids, out_slots, in_ids, in_slots, t, tile_vecs, tid);
        V vi[U], vo[U];
        if (s1 > s0) {
            const LaneTile<V> lo =
                lane_tile<V, false, true>(p, out_ids, out_slots, in_ids, in_slots, s0, tile_vecs, tid);
            tile_loads<V, U, true, false>(li, lanes, vi, vo);
            tile_loads<V, U, false, true>(lo, lanes, vi, vo);
            tile_stores<V, U, false, true>(lo, lanes, vi, vo);
            tile_stores<V, U, true, false>(li, lanes, vi, vo);
        } else {
            tile_loads<V, U, true, false>(li, lanes, vi, vo);
            tile_stores<V, U, true, false>(li, lanes, vi, vo);
        }
    }
}

// One tile with per-lane range checks: only for shapes whose segments are not
// a whole number of tiles.
template <typename V, int U>
__device__ __forceinline__ void tile_ragged(const MoveParams &p, const int32_t *__restrict__ out_ids,
                                            const int32_t *__restrict__ out_slots,
                                            const int32_t *__restrict__ in_ids,
                                            const int32_t *__restrict__ in_slots, uint32_t t, uint32_t lanes,
                                            uint32_t tid)
{
    const uint32_t tile_vecs = lanes * U;
    const bool do_in = t < p.in.tiles, do_out = t < p.out.tiles;
    const uint32_t v0 = (t % p.tiles_per_seg) * tile_vecs + tid;
    V vi[U], vo[U];
    if (do_in) {
        const LaneTile<V> a = lane_tile<V, true, false>(p, out_ids, out_slots, in_ids, in_slots, t, tile_vecs, tid);
#pragma unroll
        for (int u = 0; u < U; u++)
            if (v0 + u * lanes < p.vec_per_seg) vi[u] = a.src_i[u * lanes];
#pragma unroll
        for (int u = 0; u < U; u++)
            if (v0 + u * lanes < p.vec_per_seg) a.dst_i[u * lanes] = vi[u];
    }
    if (do_out) {
        const LaneTile<V> a = lane_tile<V, false, true>(p, out_ids, out_slots, in_ids, in_slots, t, tile_vecs, tid);
#pragma unroll
        for (int u = 0; u < U; u++)
            if (v0 + u * lanes < p.vec_per_seg) vo[u] = a.src_o[u * lanes];
#pragma unroll
        for (int u = 0; u < U; u++)
            if (v0 + u * lanes < p.vec_per_seg) a.dst_o[u * lanes] = vo[u];
    }
}

// V: vector moved per lane (16 bytes when the segment allows it).
// U: vectors per lane per tile; a tile is blockDim.x * U consecutive vectors of
//    one segment, so every wave touches 64 * sizeof(V) contiguous bytes per
//    access on both sides (full 1 KiB rows at V = 16 bytes).
// Workgroup g takes tiles g, g + G, ... .  Tile index t means tile t of the out
// list and tile t of the in list: while both lists last, every lane alternates
// an out-vector with an in-vector, which locks the two link directions 1:1;
// the longer list's remainder then runs alone.  Lists may be empty.  With
// mix_q set (in list longer, full tiles) the out tiles are instead spread over
// the whole in list.
template <typename V, int U>
__global__ __launch_bounds__(kMaxThreads) void kv_move_kernel(const MoveParams p,
                                                              const int32_t *__restrict__ out_ids,
                                                              const int32_t *__restrict__ out_slots,
                                                              const int32_t *__restrict__ in_ids,
                                                              const int32_t *__restrict__ in_slots)
{
    const uint32_t tid = threadIdx.x, lanes = blockDim.x, stride = gridDim.x;
    const uint32_t n_both = p.out.tiles < p.in.tiles ? p.out.tiles : p.in.tiles;
    const uint32_t n_all = p.out.tiles > p.in.tiles ? p.out.tiles : p.in.tiles;
    uint32_t t = blockIdx.x;
    if (!p.full_tiles) {
        for (; t < n_all; t += stride) tile_ragged<V, U>(p, out_ids, out_slots, in_ids, in_slots, t, lanes, tid);
        return;
    }
    if (p.mix_q) {
        run_in_heavy<V, U>(p, out_ids, out_slots, in_ids, in_slots, t, stride, lanes, tid);
        return;
    }
    t = run_full<V, U, true, true>(p, out_ids, out_slots, in_ids, in_slots, t, n_both, stride, lanes, tid);
    if (p.out.tiles > p.in.tiles)
        run_full<V, U, false, true>(p, out_ids, out_slots, in_ids, in_slots, t, n_all, stride, lanes, tid);
    else
        run_full<V, U, true, false>(p, out_ids, out_slots, in_ids, in_slots, t, n_all, stride, lanes, tid);
}

// Synthetic decode reader: streams every segment of the named blocks, plane by
// plane (layer-major, as attention over the running requests would), and adds
// up all 32-bit words modulo 2^64.  HBM-bound; read-only.  One tile is
// kThreads * U 16-byte vectors of one segment.  Persistent workgroups claim
// runs of kReadClaim tiles from a counter, in tile order, so at any moment the
// chip streams one contiguous front of the cache, and a CU that is slowed by a
// co-running kernel simply claims less (with a fixed share per workgroup the
// slowest CU sets the pace of the whole pass).  One short-lived workgroup per
// few tiles, left to the hardware dispatcher, measured 27 % slower.
struct ReadParams {
    const uint8_t *hbm;
    const int32_t *ids;
    unsigned long long *acc;  // one 64-bit accumulator in device memory
    uint64_t hbm_block_stride;
    uint64_t hbm_plane_stride;
    uint32_t n;              // blocks
    uint32_t n_planes;
    uint32_t vec_per_seg;    // seg_bytes / 16
    uint32_t tiles_per_seg;
    uint32_t tiles;          // n * n_planes * tiles_per_seg
    unsigned int *next;      // tile counter of this pass, zero at launch
};

constexpr uint32_t kReadClaim = 4;  // tiles a workgroup claims per turn

template <int U>
__global__ __launch_bounds__(kThreads) void kv_reader_kernel(const ReadParams p)
{
    const uint32_t tid = threadIdx.x;
    unsigned long long sum = 0;
    __shared__ uint32_t claimed;
    for (;;) {
        if (tid == 0) claimed = atomicAdd(p.next, kReadClaim);
        __syncthreads();
        const uint32_t t0 = claimed;
        __syncthreads();
        if (t0 >= p.tiles) break;
        const uint32_t t1 = min(p.tiles, t0 + kReadClaim);
        for (uint32_t t = t0; t < t1; t++) {
        const uint32_t segidx = t / p.tiles_per_seg;
        const uint32_t tin = t - segidx * p.tiles_per_seg;
        const uint32_t pl = segidx / p.n;
        const uint32_t i = segidx - pl * p.n;
        const u32x4 *src = reinterpret_cast<const u32x4 *>(
            p.hbm + (uint64_t)pl * p.hbm_plane_stride + (uint64_t)(uint32_t)p.ids[i] * p.hbm_block_stride);
        const uint32_t v0 = tin * (kThreads * U) + tid;
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; u++) {
            const uint32_t vi = v0 + u * kThreads;
            v[u] = vi < p.vec_per_seg ? src[vi] : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < U; u++)
            sum += (unsigned long long)v[u].x + v[u].y + (unsigned long long)v[u].z + v[u].w;
        }
    }
    // wave reduction, then one atomic per wave
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_down(sum, off, 64);
    if ((tid & 63u) == 0) atomicAdd(p.acc, sum);
}

}  // namespace dkv
