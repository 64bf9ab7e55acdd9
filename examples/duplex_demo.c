/*
 * DuplexKV through its C ABI alone: no Python, no PyTorch.
 *
 * Allocates a Llama-3-8B-shaped paged KV cache in HBM, fills it with a seeded
 * byte pattern, swaps one request's blocks out to the pinned pool while another
 * request's blocks come in (the duplex rotation of Section 4.3.2 of the paper),
 * checks every moved block on the CPU, and prints the rates.
 *
 * Build (from the repository root, after building the library), with any C compiler:
 *   gcc -O2 examples/duplex_demo.c -Iinclude -I/opt/rocm/include -Lpaper_2601_20309_amd -lduplexkv \
 *       -L/opt/rocm/lib -lamdhip64 -Wl,-rpath,$PWD/paper_2601_20309_amd -Wl,-rpath,/opt/rocm/lib \
 *       -o examples/duplex_demo
 * (the HIP runtime is only used here to allocate and fill the cache).
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "duplexkv.h"

#define CHECK_HIP(x)                                                                       \
    do {                                                                                   \
        hipError_t e_ = (x);                                                               \
        if (e_ != hipSuccess) {                                                            \
            fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));                 \
            return 2;                                                                      \
        }                                                                                  \
    } while (0)
#define CHECK_KV(x)                                                                        \
    do {                                                                                   \
        int r_ = (x);                                                                      \
        if (r_ != KV_OK) {                                                                 \
            fprintf(stderr, "%s failed: %s\n", #x, kv_strerror(r_));                       \
            return 3;                                                                      \
        }                                                                                  \
    } while (0)

/* byte b of (plane, block): a pattern that differs between any two segments */
static uint8_t pattern(uint32_t plane, uint32_t block, uint64_t b)
{
    uint64_t x = ((uint64_t)plane << 40) ^ ((uint64_t)block << 20) ^ b;
    x ^= x >> 33; x *= 0xff51afd7ed558ccdULL; x ^= x >> 29;
    return (uint8_t)x;
}

int main(int argc, char **argv)
{
    const int32_t n_move = argc > 1 ? atoi(argv[1]) : 128;   /* blocks each way */
    kv_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.n_layers = 32, cfg.n_kv_heads = 8, cfg.head_dim = 128, cfg.block_size = 16, cfg.elem_bytes = 2;
    cfg.n_hbm_blocks = 1024, cfg.n_host_slots = 512;
    cfg.host_layout = KV_HOST_BLOCK_FIRST, cfg.path = KV_PATH_AUTO, cfg.hbm_layout = KV_HBM_LAYER_FIRST;
    if (n_move < 1 || 2 * n_move > cfg.n_host_slots || 2 * n_move > cfg.n_hbm_blocks) {
        fprintf(stderr, "blocks each way must be 1..%d\n", cfg.n_host_slots / 2);
        return 1;
    }
    const uint64_t seg = kv_seg_bytes(&cfg), blk = kv_block_bytes(&cfg), cache_bytes = kv_cache_bytes(&cfg);
    const uint32_t planes = 2u * (uint32_t)cfg.n_layers;
    printf("segment %llu B, block %llu B, cache %.2f GiB, pool %.2f GiB\n", (unsigned long long)seg,
           (unsigned long long)blk, cache_bytes / 1073741824.0, kv_pool_bytes(&cfg) / 1073741824.0);

    /* the cache: [layer][K|V][block][...], filled on the host and copied up */
    uint8_t *image = malloc(cache_bytes);
    if (!image) return 1;
    for (uint32_t pl = 0; pl < planes; pl++)
        for (uint32_t b = 0; b < (uint32_t)cfg.n_hbm_blocks; b++) {
            uint8_t *s = image + ((uint64_t)pl * cfg.n_hbm_blocks + b) * seg;
            for (uint64_t k = 0; k < seg; k += 64) s[k] = pattern(pl, b, k);   /* one byte per 64 is enough to tell */
        }
    void *cache = NULL;
    CHECK_HIP(hipMalloc(&cache, cache_bytes));
    CHECK_HIP(hipMemcpy(cache, image, cache_bytes, hipMemcpyHostToDevice));

    kv_engine *eng = NULL;
    CHECK_KV(kv_create(&eng, &cfg, cache, NULL, NULL, NULL));
    void *pool_v = NULL;
    uint64_t pool_bytes = 0;
    CHECK_KV(kv_host_pool(eng, &pool_v, &pool_bytes));
    uint8_t *pool = pool_v;

    /* request A: blocks 3, 10, 17, ... leave to slots 0..n-1; request B waits in slots
     * n..2n-1 (staged here with the pattern of blocks that do not exist in the cache) and
     * comes back into blocks 5, 12, 19, ... */
    int32_t *oi = malloc(4 * (size_t)n_move * sizeof(int32_t)), *os = oi + n_move, *ii = os + n_move, *is = ii + n_move;
    for (int32_t k = 0; k < n_move; k++) {
        oi[k] = (3 + 7 * k) % cfg.n_hbm_blocks, os[k] = k;
        ii[k] = (5 + 7 * k) % cfg.n_hbm_blocks, is[k] = n_move + k;
        for (uint32_t pl = 0; pl < planes; pl++) {
            uint8_t *s = pool + (uint64_t)is[k] * blk + (uint64_t)pl * seg;   /* block-first pool */
            for (uint64_t b = 0; b < seg; b += 64) s[b] = pattern(pl, 100000u + (uint32_t)k, b);
        }
    }
    CHECK_KV(kv_validate(&cfg, oi, os, n_move, ii, is, n_move));

    double d2h, h2d, d2h_b, h2d_b;
    CHECK_KV(kv_probe_link(256ull << 20, 5, &d2h, &h2d, &d2h_b, &h2d_b));
    printf("hipMemcpyAsync pinned: D2H %.2f, H2D %.2f GB/s; both at once %.2f per direction\n", d2h, h2d, d2h_b);

    /* rotate, check, rotate back, ... ; time the last few */
    kv_stats st;
    double best = 1e30;
    for (int it = 0; it < 8; it++) {
        if (it % 2 == 0) CHECK_KV(kv_rotate(eng, oi, os, n_move, ii, is, n_move));
        else CHECK_KV(kv_rotate(eng, ii, is, n_move, oi, os, n_move));   /* the inverse */
        CHECK_KV(kv_wait(eng));
        CHECK_KV(kv_last_stats(eng, &st));
        if (it >= 2 && st.ms_e2e < best) best = st.ms_e2e;
        if (it == 0) {
            /* slots 0..n-1 now hold A's blocks; B's blocks are in the cache */
            CHECK_HIP(hipMemcpy(image, cache, cache_bytes, hipMemcpyDeviceToHost));
            uint64_t bad = 0;
            for (int32_t k = 0; k < n_move; k++)
                for (uint32_t pl = 0; pl < planes; pl++)
                    for (uint64_t b = 0; b < seg; b += 64) {
                        bad += pool[(uint64_t)os[k] * blk + (uint64_t)pl * seg + b] != pattern(pl, (uint32_t)oi[k], b);
                        bad += image[((uint64_t)pl * cfg.n_hbm_blocks + ii[k]) * seg + b] !=
                               pattern(pl, 100000u + (uint32_t)k, b);
                    }
            if (bad) {
                fprintf(stderr, "%llu bytes differ after the rotation\n", (unsigned long long)bad);
                return 4;
            }
            printf("rotation verified on the CPU: %d blocks out, %d in\n", n_move, n_move);
        }
    }
    const double moved = 2.0 * n_move * (double)blk;
    printf("duplex rotation: %.3f ms, %.2f GB/s both ways (%.1f %% / %.1f %% of the one-way peaks at once), path %d, %d launch(es)\n",
           best, moved / best / 1e6, 100.0 * moved / 2 / best / 1e6 / d2h, 100.0 * moved / 2 / best / 1e6 / h2d,
           st.path_used, st.n_launches);

    /* The same rotation once more through the entry point that allocates nothing: no
     * engine, just the configuration, the two buffers and a stream (the engine is idle and
     * its pool is pinned memory like any other).  After an even number of steps A is back
     * in the cache and B in its slots, so the outcome must be the one checked above. */
    CHECK_KV(kv_rotate_static(&cfg, cache, pool, NULL, oi, os, n_move, ii, is, n_move));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(image, cache, cache_bytes, hipMemcpyDeviceToHost));
    {
        uint64_t bad = 0;
        for (int32_t k = 0; k < n_move; k++)
            for (uint32_t pl = 0; pl < planes; pl++)
                for (uint64_t b = 0; b < seg; b += 64) {
                    bad += pool[(uint64_t)os[k] * blk + (uint64_t)pl * seg + b] != pattern(pl, (uint32_t)oi[k], b);
                    bad += image[((uint64_t)pl * cfg.n_hbm_blocks + ii[k]) * seg + b] != pattern(pl, 100000u + (uint32_t)k, b);
                }
        if (bad) {
            fprintf(stderr, "%llu bytes differ after kv_rotate_static\n", (unsigned long long)bad);
            return 5;
        }
        printf("kv_rotate_static verified on the CPU\n");
    }
    CHECK_KV(kv_destroy(eng));
    CHECK_HIP(hipFree(cache));
    free(image);
    free(oi);
    return 0;
}
