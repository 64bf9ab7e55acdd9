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

constexpr int kThreads = 256;  // 4 waves per workgroup

// One direction's block list as the kernel sees it.
struct DirDesc {
    const int32_t *ids;    // HBM block ids, device-readable
    const int32_t *slots;  // far-side slots; nullptr = slot i is list index i
    uint32_t n;            // blocks
    uint32_t tiles;        // n * n_planes * tiles_per_seg
};

// Addressing (Section 4.3.1 of the paper: layer x block x segment):
//   HBM  segment (plane, id)   at hbm + plane * hbm_plane_stride + id * seg_bytes
//   far  segment (plane, slot) at far + slot * far_slot_stride + plane * far_plane_stride
// `plane` = layer * 2 + (0 for K, 1 for V).
struct MoveParams {
    uint8_t *hbm;
    uint8_t *far_out;  // destination of the out direction (host pool or staging)
    uint8_t *far_in;   // source of the in direction
    uint64_t seg_bytes;
    uint64_t hbm_plane_stride;
    uint64_t far_slot_stride_out, far_plane_stride_out;
    uint64_t far_slot_stride_in, far_plane_stride_in;
    uint32_t plane0;         // first plane this launch covers
    uint32_t n_planes;       // planes this launch covers
    uint32_t vec_per_seg;    // seg_bytes / sizeof(V)
    uint32_t tiles_per_seg;  // ceil(vec_per_seg / (kThreads * U))
    uint32_t plane_major;    // tile order: 1 = [plane][i][tile], 0 = [i][plane][tile]
    DirDesc out, in;
};

// HBM-side accesses: every byte is touched once, so NT = true marks them
// non-temporal (no reuse worth keeping in L2 / MALL).
template <bool NT, typename V>
__device__ __forceinline__ V ld_hbm(const V *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT, typename V>
__device__ __forceinline__ void st_hbm(V *p, V v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// Tile t of direction d -> byte offsets of its segment and first vector index.
__device__ __forceinline__ void locate(const MoveParams &p, const DirDesc &d, uint32_t t,
                                       uint64_t slot_stride, uint64_t plane_stride,
                                       uint64_t &hbm_off, uint64_t &far_off, uint32_t &v0,
                                       uint32_t tile_vecs)
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
    const uint32_t id = (uint32_t)d.ids[i];
    const uint32_t slot = d.slots ? (uint32_t)d.slots[i] : i;
    hbm_off = (uint64_t)pl * p.hbm_plane_stride + (uint64_t)id * p.seg_bytes;
    far_off = (uint64_t)slot * slot_stride + (uint64_t)pl * plane_stride;
    v0 = tin * tile_vecs;
}

// V: vector moved per lane (16 bytes when the segment allows it).
// U: vectors per lane per tile; a tile is kThreads * U consecutive vectors of
//    one segment, so every wave touches 64 * sizeof(V) contiguous bytes per
//    access on both sides (full 1 KiB rows at V = 16 bytes).
// Workgroup g takes tiles g, g + G, ... of BOTH directions; a direction that
// has run out of tiles is simply skipped, so the lists may differ in length or
// be empty.
template <typename V, int U, bool NT>
__global__ __launch_bounds__(kThreads) void kv_move_kernel(const MoveParams p)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t tile_vecs = kThreads * U;
    const uint32_t n_tiles = p.out.tiles > p.in.tiles ? p.out.tiles : p.in.tiles;
    for (uint32_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const bool do_in = t < p.in.tiles;
        const bool do_out = t < p.out.tiles;
        V vi[U], vo[U];
        const V *src_i = nullptr, *src_o = nullptr;
        V *dst_i = nullptr, *dst_o = nullptr;
        uint32_t v0_i = 0, v0_o = 0;
        if (do_in) {
            uint64_t ho, fo;
            locate(p, p.in, t, p.far_slot_stride_in, p.far_plane_stride_in, ho, fo, v0_i, tile_vecs);
            src_i = reinterpret_cast<const V *>(p.far_in + fo);
            dst_i = reinterpret_cast<V *>(p.hbm + ho);
        }
        if (do_out) {
            uint64_t ho, fo;
            locate(p, p.out, t, p.far_slot_stride_out, p.far_plane_stride_out, ho, fo, v0_o, tile_vecs);
            src_o = reinterpret_cast<const V *>(p.hbm + ho);
            dst_o = reinterpret_cast<V *>(p.far_out + fo);
        }
        // far-side (host) loads first: they have the long latency
        if (do_in) {
#pragma unroll
            for (int u = 0; u < U; u++) {
                const uint32_t v = v0_i + u * kThreads + tid;
                if (v < p.vec_per_seg) vi[u] = src_i[v];
            }
        }
        if (do_out) {
#pragma unroll
            for (int u = 0; u < U; u++) {
                const uint32_t v = v0_o + u * kThreads + tid;
                if (v < p.vec_per_seg) vo[u] = ld_hbm<NT>(src_o + v);
            }
#pragma unroll
            for (int u = 0; u < U; u++) {
                const uint32_t v = v0_o + u * kThreads + tid;
                if (v < p.vec_per_seg) dst_o[v] = vo[u];
            }
        }
        if (do_in) {
#pragma unroll
            for (int u = 0; u < U; u++) {
                const uint32_t v = v0_i + u * kThreads + tid;
                if (v < p.vec_per_seg) st_hbm<NT>(dst_i + v, vi[u]);
            }
        }
    }
}

// Synthetic decode reader: streams every segment of the named blocks, plane by
// plane (layer-major, as attention over the running requests would), and adds
// up all 32-bit words modulo 2^64.  HBM-bound; read-only.  One tile is
// kThreads * U 16-byte vectors of one segment; tiles are dealt round-robin so
// neighbouring workgroups (which sit on different XCDs) stream neighbouring
// 4 KiB * U pieces and every HBM channel stays busy.
struct ReadParams {
    const uint8_t *hbm;
    const int32_t *ids;
    unsigned long long *acc;  // one 64-bit accumulator in device memory
    uint64_t seg_bytes;
    uint64_t hbm_plane_stride;
    uint32_t n;              // blocks
    uint32_t n_planes;
    uint32_t vec_per_seg;    // seg_bytes / 16
    uint32_t tiles_per_seg;
    uint32_t tiles;          // n * n_planes * tiles_per_seg
};

template <int U>
__global__ __launch_bounds__(kThreads) void kv_reader_kernel(const ReadParams p)
{
    const uint32_t tid = threadIdx.x;
    unsigned long long sum = 0;
    for (uint32_t t = blockIdx.x; t < p.tiles; t += gridDim.x) {
        const uint32_t segidx = t / p.tiles_per_seg;
        const uint32_t tin = t - segidx * p.tiles_per_seg;
        const uint32_t pl = segidx / p.n;
        const uint32_t i = segidx - pl * p.n;
        const u32x4 *src = reinterpret_cast<const u32x4 *>(
            p.hbm + (uint64_t)pl * p.hbm_plane_stride + (uint64_t)(uint32_t)p.ids[i] * p.seg_bytes);
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
    // wave reduction, then one atomic per wave
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_down(sum, off, 64);
    if ((tid & 63u) == 0) atomicAdd(p.acc, sum);
}

}  // namespace dkv
