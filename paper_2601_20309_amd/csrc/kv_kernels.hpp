// Device kernels of the KV rotation engine (gfx950, wave64).
//
// Everything here is data movement: no MFMA, no arithmetic beyond addressing.
// One kernel family, kv_move_kernel, serves every use:
//   - duplex rotation in ONE launch: each lane alternates a 16-byte move
//     HBM->host with a 16-byte move host->HBM, which keeps the two PCIe
//     directions locked 1:1 (measured faster in duplex than two independent
//     kernels, and above the DMA engines' duplex rate);
//   - a single direction (the other list empty): zero-copy swap-out or swap-in;
//   - pack / unpack between the scattered cache and a contiguous staging
//     buffer in HBM (the "far" side is then device memory, slot = list index)
//     when the launch is capped to a few workgroups; uncapped, pack / unpack
//     have a kernel of their own, kv_stage_kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dkv {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;          // a wave is the unit of work: one tile at a time
constexpr int kThreads = 256;      // lanes per workgroup of the HBM-bound launches and of the reader (4 waves)
constexpr int kMaxThreads = 1024;  // workgroups only pack waves; any multiple of 64 up to this

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
    uint32_t tiles_per_seg;  // ceil(vec_per_seg / (64 * U))
    uint32_t plane_major;    // tile order: 1 = [plane][i][tile], 0 = [i][plane][tile]
    uint32_t full_tiles;     // 1: vec_per_seg is a multiple of the tile, no lane is ever out of range
    // 0, or ceil(out.tiles * 2^32 / in.tiles) when the in list is the longer one and
    // the out tiles are to be spread evenly over it (see make_job)
    uint64_t mix_q;
    // nullptr: wave w of W takes tiles w, w + W, ...; else two counters in device
    // memory, zero at launch, [0] the next unclaimed tile, [1] the waves that are done
    unsigned int *claim;
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

// What one wave does in one step: an in tile, an out tile, or one of each.
// Everything in it is uniform over the wave except the lane's own pointers.
template <typename V>
struct Job {
    const V *src_i;
    V *dst_i;
    const V *src_o;
    V *dst_o;
    uint32_t do_in, do_out;
    // this lane's first vector within the segment, per direction (range checks of
    // ragged tiles; the two differ when the out tiles are spread over the in tiles)
    uint32_t v0_i, v0_o;
};

// Step t of a launch.  Normally step t is tile t of the out list and tile t of
// the in list, as far as each list goes: while both last, every lane alternates
// an out-vector with an in-vector, which locks the two link directions 1:1, and
// the longer list's remainder then runs alone.
//
// With mix_q set the in list is the longer one: its tiles set the pace and the
// out tiles are spread evenly over them, out tile s riding with the in tile t
// at which floor(t * q / 2^32) steps from s to s + 1 (q = ceil(S * 2^32 / L), so
// the steps are 0 or 1 and all S out tiles are met exactly once over the L in
// tiles).  Measured on PCIe Gen5 x16: host->HBM reads can stay at the link's
// one-way rate (55-57 GB/s) while up to ~0.85 as many bytes go the other way
// (47 GB/s), 102 GB/s in all, whereas pairing the lists 1:1 and moving the rest
// of the in list afterwards holds both at 49.5 GB/s for the paired part.  (The
// mirror case gains nothing: with the out list longer, what limits is the
// upstream direction, which carries the out data and the read requests of the
// in data, and that sum does not depend on the order.)
template <typename V, int U>
__device__ __forceinline__ Job<V> make_job(const MoveParams &p, const int32_t *__restrict__ out_ids,
                                           const int32_t *__restrict__ out_slots,
                                           const int32_t *__restrict__ in_ids,
                                           const int32_t *__restrict__ in_slots, uint32_t t, uint32_t lane)
{
    constexpr uint32_t tile_vecs = kWave * U, tile_bytes = tile_vecs * (uint32_t)sizeof(V);
    Job<V> j{nullptr, nullptr, nullptr, nullptr, 0u, 0u, 0u, 0u};
    uint32_t t_out = t;
    if (p.mix_q) {
        const uint64_t a = (uint64_t)t * p.mix_q, b = a + p.mix_q;
        const uint32_t s0 = (uint32_t)(a >> 32);
        uint32_t s1 = (uint32_t)(b >> 32);
        s1 = s1 < p.out.tiles ? s1 : p.out.tiles;
        j.do_in = 1u;
        j.do_out = s1 > s0 ? 1u : 0u;
        t_out = s0;
    } else {
        j.do_in = t < p.in.tiles ? 1u : 0u;
        j.do_out = t < p.out.tiles ? 1u : 0u;
    }
    j.v0_i = (t % p.tiles_per_seg) * tile_vecs + lane;
    j.v0_o = p.mix_q ? (t_out % p.tiles_per_seg) * tile_vecs + lane : j.v0_i;
    if (j.do_in) {
        uint64_t ho, fo;
        locate(p, p.in, in_ids, in_slots, t, p.far_slot_stride_in, p.far_plane_stride_in, tile_bytes, ho, fo);
        j.src_i = reinterpret_cast<const V *>(p.far_in + fo) + lane;
        j.dst_i = reinterpret_cast<V *>(p.hbm + ho) + lane;
    }
    if (j.do_out) {
        uint64_t ho, fo;
        locate(p, p.out, out_ids, out_slots, t_out, p.far_slot_stride_out, p.far_plane_stride_out, tile_bytes, ho,
               fo);
        j.src_o = reinterpret_cast<const V *>(p.hbm + ho) + lane;
        j.dst_o = reinterpret_cast<V *>(p.far_out + fo) + lane;
    }
    return j;
}

// Loads of one job: the far-side (host) loads first, they have the long
// latency; then the HBM loads.  FULL: the segment is a whole number of tiles, no
// lane is ever out of range, and all loads issue back to back.  In an HBM-bound
// launch (pack / unpack, !LINK) loads and stores alike are marked non-temporal:
// nothing a mover touches is touched twice.
template <typename V, int U, bool LINK, bool FULL>
__device__ __forceinline__ void job_loads(const MoveParams &p, const Job<V> &j, V (&vi)[U], V (&vo)[U])
{
    if (j.do_in) {
#pragma unroll
        for (int u = 0; u < U; u++) {
            if (FULL || j.v0_i + u * kWave < p.vec_per_seg) {
                if constexpr (LINK) vi[u] = j.src_i[u * kWave];
                else vi[u] = __builtin_nontemporal_load(j.src_i + u * kWave);
            }
        }
    }
    if (j.do_out) {
#pragma unroll
        for (int u = 0; u < U; u++) {
            if (FULL || j.v0_o + u * kWave < p.vec_per_seg) {
                if constexpr (LINK) vo[u] = j.src_o[u * kWave];
                else vo[u] = __builtin_nontemporal_load(j.src_o + u * kWave);
            }
        }
    }
}

// Stores of one job.  Stores to the far side are marked non-temporal, and so
// are the stores into the cache of an HBM-bound launch (unpack).
// LINK (far side = host memory): plain stores linger in the write-back L2 and
// are only pushed out when evicted or when the kernel ends, so the upstream
// link idles early and a kernel's last megabytes leave while the downstream
// link idles (measured, 8 + 8 MiB both ways: 237 us plain, 188 us non-temporal).
// Pack / unpack (both sides HBM), one 256 MiB chunk whose source is in no cache:
// plain loads and stores 109 us, non-temporal stores 100 us, non-temporal loads
// and stores 95 us (HIP events around the launch).
template <typename V, int U, bool LINK, bool FULL>
__device__ __forceinline__ void job_stores(const MoveParams &p, const Job<V> &j, const V (&vi)[U],
                                           const V (&vo)[U])
{
    if (j.do_out) {
#pragma unroll
        for (int u = 0; u < U; u++)
            if (FULL || j.v0_o + u * kWave < p.vec_per_seg) __builtin_nontemporal_store(vo[u], j.dst_o + u * kWave);
    }
    if (j.do_in) {
#pragma unroll
        for (int u = 0; u < U; u++) {
            if (FULL || j.v0_i + u * kWave < p.vec_per_seg) {
                if constexpr (LINK) j.dst_i[u * kWave] = vi[u];
                else __builtin_nontemporal_store(vi[u], j.dst_i + u * kWave);
            }
        }
    }
}

// One draw of `n` consecutive steps from the counter by the wave's first lane
// (the others get 0).  The value comes back a memory latency later; drawn()
// reads it.
__device__ __forceinline__ uint32_t draw(const MoveParams &p, uint32_t lane, uint32_t n)
{
    uint32_t d = 0;
    if (lane == 0) d = atomicAdd(&p.claim[0], n);
    return d;
}

// The drawn value, wave-uniform.  The empty asm pins the first use of the
// register to this point of the program: without it the compiler is free to
// read the value (and so to wait for the atomic and for every vector memory
// access issued before it) right behind the draw.
__device__ __forceinline__ uint32_t drawn(uint32_t d)
{
    asm volatile("" : "+v"(d));
    return __builtin_amdgcn_readfirstlane(d);
}

// Fixed share: wave w of W takes steps w, w + W, ...
template <typename V, int U, bool LINK, bool FULL>
__device__ __forceinline__ void run_fixed(const MoveParams &p, const int32_t *__restrict__ out_ids,
                                          const int32_t *__restrict__ out_slots,
                                          const int32_t *__restrict__ in_ids,
                                          const int32_t *__restrict__ in_slots, uint32_t n_steps, uint32_t wave,
                                          uint32_t n_waves, uint32_t lane)
{
    uint32_t t = wave;
    if (t >= n_steps) return;
    V vi[U], vo[U];
    Job<V> cur = make_job<V, U>(p, out_ids, out_slots, in_ids, in_slots, t, lane);
    for (;;) {
        job_loads<V, U, LINK, FULL>(p, cur, vi, vo);
        t += n_waves;
        const bool more = t < n_steps;
        Job<V> nxt = cur;
        if (more) nxt = make_job<V, U>(p, out_ids, out_slots, in_ids, in_slots, t, lane);
        job_stores<V, U, LINK, FULL>(p, cur, vi, vo);
        if (!more) break;
        cur = nxt;
    }
}

// Drawn steps.  A draw takes kDrawChunk consecutive steps (one atomic per step
// would be ~50 M a second on one address, which beside an HBM-bound kernel is
// what limits the launch: 93 GB/s whatever the number of waves), except near the
// end, where steps are drawn singly so that the waves still finish within one
// step of each other.  The draw for the next chunk is issued when the current
// chunk starts and read when it ends.  Every draw the wave issues is read back
// before the function returns.
constexpr uint32_t kDrawChunk = 4;

template <typename V, int U, bool LINK, bool FULL>
__device__ __forceinline__ void run_drawn(const MoveParams &p, const int32_t *__restrict__ out_ids,
                                          const int32_t *__restrict__ out_slots,
                                          const int32_t *__restrict__ in_ids,
                                          const int32_t *__restrict__ in_slots, uint32_t n_steps, uint32_t n_waves,
                                          uint32_t lane)
{
    // steps at or beyond `single` are drawn one at a time
    const uint32_t tail = 2u * kDrawChunk * n_waves, single = n_steps > tail ? n_steps - tail : 0u;
    uint32_t c = single ? kDrawChunk : 1u;
    uint32_t t = drawn(draw(p, lane, c));  // current step
    uint32_t e = t + c;                    // end of the chunk it belongs to
    uint32_t cn = t < single ? kDrawChunk : 1u;
    uint32_t d = draw(p, lane, cn);        // the next chunk, in flight
    if (t < n_steps) {
        V vi[U], vo[U];
        Job<V> cur = make_job<V, U>(p, out_ids, out_slots, in_ids, in_slots, t, lane);
        for (;;) {
            job_loads<V, U, LINK, FULL>(p, cur, vi, vo);
            // The next step.  At the end of a chunk the pending draw is read: here,
            // where the loads have to be waited for anyway (the draw is older than
            // they are), and before the stores: the vector memory counter retires in
            // order, so reading it behind the stores would wait for them, and a wave
            // would then pay store latency and load latency in turn.  As it is, a
            // step's stores have the whole next step to retire.
            uint32_t tn = t + 1u;
            if (tn >= e) {
                tn = drawn(d);
                e = tn + cn;
                cn = tn < single ? kDrawChunk : 1u;
                d = draw(p, lane, cn);
            }
            const bool more = tn < n_steps;
            Job<V> nxt = cur;
            if (more) nxt = make_job<V, U>(p, out_ids, out_slots, in_ids, in_slots, tn, lane);
            job_stores<V, U, LINK, FULL>(p, cur, vi, vo);
            if (!more) break;
            cur = nxt;
            t = tn;
        }
    }
    (void)drawn(d);
}

// V: vector moved per lane (16 bytes when the segment allows it).
// U: vectors per lane per tile; a tile is 64 * U consecutive vectors of one
//    segment, so every wave access touches 64 * sizeof(V) contiguous bytes on
//    both sides (full 1 KiB rows at V = 16 bytes).
// LINK: the far side is host memory.
// A wave is the unit of work: it takes a step, issues its loads, works out the
// addresses of its next step (two divisions, the scalar loads of id and slot)
// while they are in flight, and stores.  What keeps the link busy is the number
// of waves: a second step in flight per wave buys what a second wave buys.
//
// Which step a wave takes next: with p.claim the waves draw step indices from a
// counter (the draw for the step after next is issued a whole step ahead, so
// its latency is never waited for).  With a fixed share per wave the waves of a
// link-bound launch drift apart by several per cent and the launch ends with a
// tail of ~100 us in which too few waves are left to fill the link; drawn steps
// end within one tile of each other, and the rate no longer depends on how the
// wave count divides the tile count.  The last wave to finish puts both
// counters back to zero for the next launch on the stream.  HBM-bound launches
// (pack / unpack with a cap on their workgroups; uncapped they run as
// kv_stage_kernel) move a tile in ~2 ns chip-wide, too fast for one counter, and
// use the fixed share.
template <typename V, int U, bool LINK>
__global__ __launch_bounds__(kMaxThreads) void kv_move_kernel(const MoveParams p,
                                                              const int32_t *__restrict__ out_ids,
                                                              const int32_t *__restrict__ out_slots,
                                                              const int32_t *__restrict__ in_ids,
                                                              const int32_t *__restrict__ in_slots)
{
    const uint32_t lane = threadIdx.x & (kWave - 1u), waves_per_wg = blockDim.x / kWave;
    const uint32_t wave = blockIdx.x * waves_per_wg + threadIdx.x / kWave, n_waves = gridDim.x * waves_per_wg;
    const uint32_t n_steps = p.mix_q ? p.in.tiles : (p.out.tiles > p.in.tiles ? p.out.tiles : p.in.tiles);
    if (!p.claim) {
        if (p.full_tiles)
            run_fixed<V, U, LINK, true>(p, out_ids, out_slots, in_ids, in_slots, n_steps, wave, n_waves, lane);
        else
            run_fixed<V, U, LINK, false>(p, out_ids, out_slots, in_ids, in_slots, n_steps, wave, n_waves, lane);
        return;
    }
    if (p.full_tiles)
        run_drawn<V, U, LINK, true>(p, out_ids, out_slots, in_ids, in_slots, n_steps, n_waves, lane);
    else
        run_drawn<V, U, LINK, false>(p, out_ids, out_slots, in_ids, in_slots, n_steps, n_waves, lane);
    // Every draw this wave issued has been read back, so the counter holds all of
    // its increments before the wave reports itself done; the wave that sees
    // every other one done can therefore put the counters back.
    if (lane == 0 && atomicAdd(&p.claim[1], 1u) == n_waves - 1u) {
        p.claim[0] = 0u;
        p.claim[1] = 0u;
    }
}

// Pack / unpack of the DMA-staged path when nothing caps the launch: both sides
// are HBM, so the kernel is bound by HBM bandwidth and wants the plainest shape
// there is.  One wave moves one tile of 64 vectors (1 KiB at 16-byte vectors)
// and ends; there are as many waves as tiles and the hardware dispatcher deals
// them out, four to a workgroup when packing and one to a workgroup when
// unpacking (scattered stores: 90.6 us against 95.7 for a 256 MiB chunk of 32 KiB
// segments; gathered loads prefer four: 87.8 against 91.4).  No loop, no counters, no second direction;
// loads and stores are non-temporal (nothing is touched twice).  The staging
// side is addressed by list index: segment (plane, i) at
// stage + i * slot_stride + (plane - plane0) * plane_stride.
struct StageParams {
    uint8_t *hbm, *stage;
    uint64_t hbm_plane_stride, hbm_block_stride;
    uint64_t slot_stride, plane_stride;  // staging
    uint32_t plane0, n_planes;           // planes this launch covers
    uint32_t n;                          // blocks
    uint32_t vec_per_seg, tiles_per_seg; // tiles of 64 vectors
    uint32_t tiles;                      // n * n_planes * tiles_per_seg
    uint32_t plane_major;                // tile order: 1 = [plane][i][tile], 0 = [i][plane][tile]
};

template <typename V, bool UNPACK>
__global__ __launch_bounds__(kThreads) void kv_stage_kernel(const StageParams p, const int32_t *__restrict__ ids)
{
    const uint32_t lane = threadIdx.x & (kWave - 1u);
    const uint32_t t = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (t >= p.tiles) return;
    const uint32_t segidx = t / p.tiles_per_seg, tin = t - segidx * p.tiles_per_seg;
    uint32_t i, pl;
    if (p.plane_major) {
        pl = segidx / p.n;
        i = segidx - pl * p.n;
    } else {
        i = segidx / p.n_planes;
        pl = segidx - i * p.n_planes;
    }
    const uint32_t v = tin * kWave + lane;
    if (v >= p.vec_per_seg) return;
    V *in_cache = reinterpret_cast<V *>(p.hbm + (uint64_t)(pl + p.plane0) * p.hbm_plane_stride +
                                        (uint64_t)(uint32_t)ids[i] * p.hbm_block_stride) + v;
    V *in_stage = reinterpret_cast<V *>(p.stage + (uint64_t)i * p.slot_stride + (uint64_t)pl * p.plane_stride) + v;
    if constexpr (UNPACK) __builtin_nontemporal_store(__builtin_nontemporal_load(in_stage), in_cache);
    else __builtin_nontemporal_store(__builtin_nontemporal_load(in_cache), in_stage);
}

// Synthetic decode reader: streams every segment of the named blocks, plane by
// plane (layer-major, as attention over the running requests would), and adds
// up all 32-bit words modulo 2^64.  HBM-bound; read-only.  One tile is
// kThreads * U 16-byte vectors of one segment.  Persistent workgroups claim
// runs of kReadClaim tiles from a counter, in tile order, so at any moment the
// chip streams one contiguous front of the cache, and a CU that is slowed by a
// co-running kernel simply claims less (with a fixed share per workgroup the
// slowest CU sets the pace of the whole pass).  One short-lived workgroup per
// few tiles, left to the hardware dispatcher, measured 27 % slower.  The loads
// are non-temporal (nothing is read twice): worth 3 % when the blocks come in
// random order and 16 % on the block-first cache, whose segments lie a whole
// block apart (5.54 -> 6.43 TB/s), nothing on consecutive blocks.
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

// Tiles a workgroup claims per turn.  One counter serves the whole chip, and at
// 6.5 TB/s a 32 KiB tile lasts 5 ns: measured over 37.5 GiB, 5.5 workgroups per
// CU, TB/s by claim size: 2 -> 4.65, 4 -> 6.51, 8 -> 6.65, 16 -> 6.74, 32 -> 6.68,
// 64 -> 6.62, 128 -> 6.53 (beyond 16 the pass ends more raggedly than the counter
// saves).
constexpr uint32_t kReadClaim = 16;
constexpr uint32_t kReadClaimTail = 4;  // within the last 2 * kReadClaim tiles per workgroup of a pass

template <int U>
__global__ __launch_bounds__(kThreads) void kv_reader_kernel(const ReadParams p)
{
    const uint32_t tid = threadIdx.x;
    unsigned long long sum = 0;
    __shared__ uint32_t claimed;
    // near the end of the pass the claims get short, so that the workgroups end
    // within a few tiles of each other (a long last claim on a slowed CU would
    // hold up the whole pass)
    const uint32_t tail = 2u * kReadClaim * gridDim.x, short_from = p.tiles > tail ? p.tiles - tail : 0u;
    uint32_t want = short_from ? kReadClaim : kReadClaimTail;
    for (;;) {
        if (tid == 0) claimed = atomicAdd(p.next, want);
        __syncthreads();
        const uint32_t t0 = claimed;
        __syncthreads();
        if (t0 >= p.tiles) break;
        const uint32_t t1 = min(p.tiles, t0 + want);
        want = t1 < short_from ? kReadClaim : kReadClaimTail;
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
            v[u] = vi < p.vec_per_seg ? __builtin_nontemporal_load(src + vi) : u32x4{0u, 0u, 0u, 0u};
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
