// Measurement program, not part of the library: which shape of copy kernel
// brings the pack / unpack step of the DMA-staged path closest to the HBM
// roofline?  It gathers one 256 MiB chunk of the Llama-3-8B-shaped cache (128
// scattered blocks x 64 planes, 8192 segments of 32 KiB out of a 16 GiB
// layer-first cache) into contiguous staging laid out [block][plane][segment],
// and scatters it back, with each of these kernels:
//   fixed      wave w of W takes tiles w, w + W, ...; 64 lanes x U 16-byte vectors
//              per tile.  Variants: plain accesses, non-temporal stores,
//              non-temporal loads, both; persistent waves that loop, or as many
//              waves as tiles (no loop, the hardware dispatcher deals them out).
//   lds        the same, staged through LDS (global -> LDS -> global), the
//              "LDS-staged wavefront copy"
//   wg-claim   a workgroup claims runs of R tiles from a counter (as the decode
//              reader does)
//   wave-claim a wave claims runs of R tiles from a counter
// and, for scale, with the runtime's own device-to-device copy of 256 MiB.
// Every pack result is compared with the first kernel's.  Times are HIP events
// around single launches (they include ~5 us of launch), median and minimum of
// 30; rocprofv3 --kernel-trace --stats on this program gives the bare kernels.
// Consecutive launches take different block lists (32 disjoint sets of 128
// blocks) and different staging buffers (4), so that no launch finds its source
// in the chip's 256 MB last-level cache: a loop over one chunk does, and then
// reports rates above the HBM peak.
//
// Build: hipcc --offload-arch=gfx950 -O3 (see paper_2601_20309_amd/build.py).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

#define CK(x)                                                                                    \
    do {                                                                                         \
        hipError_t e_ = (x);                                                                     \
        if (e_ != hipSuccess) {                                                                  \
            printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__);        \
            fflush(stdout);                                                                      \
            exit(2);                                                                             \
        }                                                                                        \
    } while (0)

struct Chunk {
    uint8_t *cache, *stage;
    const int32_t *ids;
    uint64_t plane_stride, seg;  // bytes
    uint32_t n, planes;          // blocks, planes
    unsigned int *counter;
};

// segment s = block j * planes + plane: where it lives in the cache and in staging
__device__ __forceinline__ void seg_ptrs(const Chunk &c, uint32_t s, uint8_t *&in_cache, uint8_t *&in_stage)
{
    const uint32_t j = s / c.planes, pl = s - j * c.planes;
    in_cache = c.cache + (uint64_t)pl * c.plane_stride + (uint64_t)(uint32_t)c.ids[j] * c.seg;
    in_stage = c.stage + (uint64_t)s * c.seg;
}

template <int U, bool NT_LOAD, bool NT_STORE>
__device__ __forceinline__ void move_tile(const u32x4 *a, u32x4 *b, uint32_t stride)
{
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; u++) v[u] = NT_LOAD ? __builtin_nontemporal_load(a + u * stride) : a[u * stride];
#pragma unroll
    for (int u = 0; u < U; u++) {
        if (NT_STORE) __builtin_nontemporal_store(v[u], b + u * stride);
        else b[u * stride] = v[u];
    }
}

template <int U, bool NT_LOAD, bool NT_STORE, bool UNPACK>
__global__ void k_fixed(const Chunk c)
{
    const uint32_t lane = threadIdx.x & 63u, wpw = blockDim.x / 64;
    const uint32_t wave = blockIdx.x * wpw + threadIdx.x / 64, n_waves = gridDim.x * wpw;
    const uint32_t tile_b = 64 * U * 16, tps = (uint32_t)(c.seg / tile_b), tiles = c.n * c.planes * tps;
    for (uint32_t t = wave; t < tiles; t += n_waves) {
        const uint32_t s = t / tps, tin = t - s * tps;
        uint8_t *pc, *ps;
        seg_ptrs(c, s, pc, ps);
        const u32x4 *a = (const u32x4 *)((UNPACK ? ps : pc) + (uint64_t)tin * tile_b) + lane;
        u32x4 *b = (u32x4 *)((UNPACK ? pc : ps) + (uint64_t)tin * tile_b) + lane;
        move_tile<U, NT_LOAD, NT_STORE>(a, b, 64);
    }
}

template <int U, bool NT_LOAD>
__global__ void k_lds(const Chunk c)
{
    extern __shared__ u32x4 lds[];
    const uint32_t lane = threadIdx.x & 63u, wpw = blockDim.x / 64, wiw = threadIdx.x / 64;
    const uint32_t wave = blockIdx.x * wpw + wiw, n_waves = gridDim.x * wpw;
    const uint32_t tile_b = 64 * U * 16, tps = (uint32_t)(c.seg / tile_b), tiles = c.n * c.planes * tps;
    u32x4 *mine = lds + wiw * 64 * U;  // a wave's own stretch of LDS: no barrier needed
    for (uint32_t t = wave; t < tiles; t += n_waves) {
        const uint32_t s = t / tps, tin = t - s * tps;
        uint8_t *pc, *ps;
        seg_ptrs(c, s, pc, ps);
        const u32x4 *a = (const u32x4 *)(pc + (uint64_t)tin * tile_b) + lane;
        u32x4 *b = (u32x4 *)(ps + (uint64_t)tin * tile_b) + lane;
#pragma unroll
        for (int u = 0; u < U; u++) mine[u * 64 + lane] = NT_LOAD ? __builtin_nontemporal_load(a + u * 64) : a[u * 64];
#pragma unroll
        for (int u = 0; u < U; u++) __builtin_nontemporal_store(mine[u * 64 + lane], b + u * 64);
    }
}

template <int U, bool NT>
__global__ void k_wg_claim(const Chunk c, uint32_t run)
{
    const uint32_t tid = threadIdx.x, tile_b = blockDim.x * U * 16, tps = (uint32_t)(c.seg / tile_b);
    const uint32_t tiles = c.n * c.planes * tps;
    __shared__ uint32_t claimed;
    for (;;) {
        if (tid == 0) claimed = atomicAdd(c.counter, run);
        __syncthreads();
        const uint32_t t0 = claimed;
        __syncthreads();
        if (t0 >= tiles) break;
        const uint32_t t1 = min(tiles, t0 + run);
        for (uint32_t t = t0; t < t1; t++) {
            const uint32_t s = t / tps, tin = t - s * tps;
            uint8_t *pc, *ps;
            seg_ptrs(c, s, pc, ps);
            move_tile<U, NT, NT>((const u32x4 *)(pc + (uint64_t)tin * tile_b) + tid,
                                          (u32x4 *)(ps + (uint64_t)tin * tile_b) + tid, blockDim.x);
        }
    }
}

template <int U>
__global__ void k_wave_claim(const Chunk c, uint32_t run)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t tile_b = 64 * U * 16, tps = (uint32_t)(c.seg / tile_b), tiles = c.n * c.planes * tps;
    uint32_t d = 0;
    if (lane == 0) d = atomicAdd(c.counter, run);
    uint32_t t0 = __builtin_amdgcn_readfirstlane(d);
    while (t0 < tiles) {
        uint32_t dn = 0;  // the next claim is in flight while this one is worked off
        if (lane == 0) dn = atomicAdd(c.counter, run);
        const uint32_t t1 = min(tiles, t0 + run);
        for (uint32_t t = t0; t < t1; t++) {
            const uint32_t s = t / tps, tin = t - s * tps;
            uint8_t *pc, *ps;
            seg_ptrs(c, s, pc, ps);
            move_tile<U, true, true>((const u32x4 *)(pc + (uint64_t)tin * tile_b) + lane,
                                      (u32x4 *)(ps + (uint64_t)tin * tile_b) + lane, 64);
        }
        t0 = __builtin_amdgcn_readfirstlane(dn);
    }
}

int main()
{
    const uint32_t NB = 8192, PL = 64, N = 128;
    const uint64_t SEG = 32768;
    const uint32_t SETS = 32, STAGES = 4;
    const size_t cache_b = (size_t)NB * PL * SEG, chunk_b = (size_t)N * PL * SEG;
    uint8_t *cache, *stages, *ref;
    int32_t *ids;
    unsigned int *counter;
    CK(hipMalloc(&cache, cache_b));
    CK(hipMalloc(&stages, STAGES * chunk_b));
    CK(hipMalloc(&ref, chunk_b));
    CK(hipMalloc(&ids, SETS * N * sizeof(int32_t)));
    CK(hipMalloc(&counter, 256));
    {  // a pattern that depends on the address
        std::vector<uint32_t> h(1 << 20);
        for (size_t i = 0; i < h.size(); i++) h[i] = (uint32_t)(i * 2654435761u);
        for (size_t off = 0; off < cache_b; off += h.size() * 4) {
            h[0] = (uint32_t)(off >> 20);
            CK(hipMemcpy(cache + off, h.data(), h.size() * 4, hipMemcpyHostToDevice));
        }
    }
    std::mt19937 rng(7);
    std::vector<int32_t> perm(NB);
    for (uint32_t i = 0; i < NB; i++) perm[i] = (int32_t)i;
    std::shuffle(perm.begin(), perm.end(), rng);
    CK(hipMemcpy(ids, perm.data(), SETS * N * sizeof(int32_t), hipMemcpyHostToDevice));
    uint8_t *stage = stages;
    Chunk c{cache, stage, ids, (uint64_t)NB * SEG, SEG, N, PL, counter};
    hipStream_t s;
    CK(hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    Chunk cr = c;
    cr.stage = ref;
    hipLaunchKernelGGL((k_fixed<4, false, false, false>), dim3(2048), dim3(256), 0, s, cr);
    CK(hipStreamSynchronize(s));
    std::vector<uint8_t> want(chunk_b), got(chunk_b);
    CK(hipMemcpy(want.data(), ref, chunk_b, hipMemcpyDeviceToHost));

    printf("| kernel | grid | result | median us | min us | TB/s read + write (median) | of 8 TB/s |\n");
    printf("|---|---|---|---|---|---|---|\n");
    // check: 1 = the staging must equal the reference gather; 0 = nothing to compare (copy / unpack)
    auto run = [&](const char *name, const char *grid, int check, auto launch) {
        const char *same = "-";
        if (check) {
            CK(hipMemsetAsync(stage, 0, chunk_b, s));
            CK(hipMemsetAsync(counter, 0, 256, s));
            launch();
            CK(hipStreamSynchronize(s));
            CK(hipMemcpy(got.data(), stage, chunk_b, hipMemcpyDeviceToHost));
            same = memcmp(got.data(), want.data(), chunk_b) == 0 ? "equal" : "DIFFERS";
        }
        std::vector<float> us;
        for (uint32_t r = 0; r < 34; r++) {
            c.ids = ids + (size_t)((r + 1) % SETS) * N;  // set 0 is the checked one
            c.stage = stages + (size_t)(r % STAGES) * chunk_b;
            CK(hipMemsetAsync(counter, 0, 256, s));
            CK(hipEventRecord(e0, s));
            launch();
            CK(hipEventRecord(e1, s));
            CK(hipEventSynchronize(e1));
            float t;
            CK(hipEventElapsedTime(&t, e0, e1));
            if (r >= 2) us.push_back(t * 1e3f);
        }
        c.ids = ids;
        c.stage = stage;
        std::sort(us.begin(), us.end());
        const double med = us[us.size() / 2], tbs = 2.0 * chunk_b / med / 1e6;
        printf("| %s | %s | %s | %.1f | %.1f | %.2f | %.0f %% |\n", name, grid, same, med, us[0], tbs, tbs / 8 * 100);
        fflush(stdout);
    };
#define FIXED(U, L, S, UNP, G, T) \
    hipLaunchKernelGGL((k_fixed<U, L, S, UNP>), dim3(G), dim3(T), 0, s, c)
    run("runtime device-to-device copy, 256 MiB contiguous", "-", 0, [&] {
        CK(hipMemcpyAsync(c.stage, cache + (size_t)(c.ids - ids) / N * 2 * chunk_b, chunk_b, hipMemcpyDeviceToDevice, s));
    });
    // persistent waves looping over 4 KiB tiles: what the hints are worth
    run("pack, waves loop over 4 KiB tiles, plain loads and stores", "2048 x 256", 1, [&] { FIXED(4, false, false, false, 2048, 256); });
    run("pack, waves loop over 4 KiB tiles, non-temporal stores", "2048 x 256", 1, [&] { FIXED(4, false, true, false, 2048, 256); });
    run("pack, waves loop over 4 KiB tiles, non-temporal loads", "2048 x 256", 1, [&] { FIXED(4, true, false, false, 2048, 256); });
    run("pack, waves loop over 4 KiB tiles, non-temporal loads and stores", "2048 x 256", 1, [&] { FIXED(4, true, true, false, 2048, 256); });
    run("pack, waves loop over 8 KiB tiles, non-temporal loads and stores", "1024 x 256", 1, [&] { FIXED(8, true, true, false, 1024, 256); });
    // the same through LDS
    run("pack, LDS-staged, 4 KiB tiles, plain loads, non-temporal stores", "2048 x 256", 1,
        [&] { hipLaunchKernelGGL((k_lds<4, false>), dim3(2048), dim3(256), 4 * 64 * 4 * 16, s, c); });
    run("pack, LDS-staged, 4 KiB tiles, non-temporal loads and stores", "2048 x 256", 1,
        [&] { hipLaunchKernelGGL((k_lds<4, true>), dim3(2048), dim3(256), 4 * 64 * 4 * 16, s, c); });
    run("pack, LDS-staged, 8 KiB tiles, non-temporal loads and stores", "1024 x 256", 1,
        [&] { hipLaunchKernelGGL((k_lds<8, true>), dim3(1024), dim3(256), 4 * 64 * 8 * 16, s, c); });
    // tiles claimed from a counter
    run("pack, workgroup claims 4 tiles of 16 KiB, plain", "1408 x 256", 1,
        [&] { hipLaunchKernelGGL((k_wg_claim<4, false>), dim3(1408), dim3(256), 0, s, c, 4u); });
    run("pack, workgroup claims 4 tiles of 16 KiB, non-temporal loads and stores", "1408 x 256", 1,
        [&] { hipLaunchKernelGGL((k_wg_claim<4, true>), dim3(1408), dim3(256), 0, s, c, 4u); });
    run("pack, workgroup claims 2 tiles of 32 KiB, non-temporal loads and stores", "1408 x 256", 1,
        [&] { hipLaunchKernelGGL((k_wg_claim<8, true>), dim3(1408), dim3(256), 0, s, c, 2u); });
    run("pack, wave claims 16 tiles of 4 KiB, non-temporal loads and stores", "1024 x 256", 1,
        [&] { hipLaunchKernelGGL((k_wave_claim<4>), dim3(1024), dim3(256), 0, s, c, 16u); });
    // no loop: as many waves as tiles, dealt out by the hardware dispatcher
    run("pack, one 4 KiB tile per wave, non-temporal loads and stores", "16384 x 256", 1, [&] { FIXED(4, true, true, false, 16384, 256); });
    run("pack, one 2 KiB tile per wave, non-temporal loads and stores", "32768 x 256", 1, [&] { FIXED(2, true, true, false, 32768, 256); });
    run("pack, one 1 KiB tile per wave, non-temporal loads and stores (the library's shape)", "65536 x 256", 1,
        [&] { FIXED(1, true, true, false, 65536, 256); });
    run("pack, one 1 KiB tile per wave, plain loads and stores", "65536 x 256", 1, [&] { FIXED(1, false, false, false, 65536, 256); });
    // the same waves, more or fewer to a workgroup
    run("pack, one 1 KiB tile per wave, one wave per workgroup", "262144 x 64", 1, [&] { FIXED(1, true, true, false, 262144, 64); });
    run("pack, one 1 KiB tile per wave, 16 waves per workgroup", "16384 x 1024", 1, [&] { FIXED(1, true, true, false, 16384, 1024); });
    run("unpack, waves loop over 4 KiB tiles, plain loads and stores", "2048 x 256", 0, [&] { FIXED(4, false, false, true, 2048, 256); });
    run("unpack, waves loop over 4 KiB tiles, non-temporal loads and stores", "2048 x 256", 0, [&] { FIXED(4, true, true, true, 2048, 256); });
    run("unpack, one 1 KiB tile per wave, non-temporal stores", "65536 x 256", 0, [&] { FIXED(1, false, true, true, 65536, 256); });
    run("unpack, one 1 KiB tile per wave, non-temporal loads and stores", "65536 x 256", 0,
        [&] { FIXED(1, true, true, true, 65536, 256); });
    run("unpack, one 1 KiB tile per wave, 16 waves per workgroup", "16384 x 1024", 0, [&] { FIXED(1, true, true, true, 16384, 1024); });
    run("unpack, one 1 KiB tile per wave, one wave per workgroup (the library's shape)", "262144 x 64", 0,
        [&] { FIXED(1, true, true, true, 262144, 64); });
    return 0;
}
