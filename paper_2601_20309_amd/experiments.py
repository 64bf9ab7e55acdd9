"""Measurements beyond bench.py's headline line, on one MI355X:

  python -m paper_2601_20309_amd.experiments ladder        # analogue of the paper's Table 2
  python -m paper_2601_20309_amd.experiments configs       # the headline, batch and long-context rotations, default path
  python -m paper_2601_20309_amd.experiments interference  # configs[4]: rotation beside a decode reader
  python -m paper_2601_20309_amd.experiments reader        # the decode reader alone (profiling target)
  python -m paper_2601_20309_amd.experiments eager         # a preemption with and without eager block rotation
  python -m paper_2601_20309_amd.experiments layouts       # layer-first against block-first cache layout
  python -m paper_2601_20309_amd.experiments linksweep     # bandwidth against segment size, copies and kernels
  python -m paper_2601_20309_amd.experiments serve         # LVF + block table + engine in a cross-iteration pipeline
  python -m paper_2601_20309_amd.experiments sizes         # rotation rate against rotation size
  python -m paper_2601_20309_amd.experiments ratio         # rates against the mix of the two directions
  python -m paper_2601_20309_amd.experiments poolkinds     # does the kind of pinned memory the pool is made of matter?
  python -m paper_2601_20309_amd.experiments layers        # kernel paths layer by layer: cost of the chunks, when layer 0 is ready
  python -m paper_2601_20309_amd.experiments chunks        # DMA-staged path against chunk size: what serial chunks cost
  python -m paper_2601_20309_amd.experiments splitcalls    # configs[2] in one call, in 32 waited calls, in 32 un-waited calls
  python -m paper_2601_20309_amd.experiments packalone     # pack and unpack kernels with nothing beside them (profiling target)
  python -m paper_2601_20309_amd.experiments packshapes    # shapes of pack / unpack kernel against the HBM roofline

Each prints a markdown table.  Correctness of every path measured here is
covered by the GPU tests; these runs only time.
"""
from __future__ import annotations

import os
import statistics
import subprocess
import sys
import time

import numpy as np
import torch

from . import binding as B
from . import workloads as W


def _cache(shape):
    # contents do not matter to a timing run; N(0,1) bf16 all the same
    c = torch.empty(shape.cache_dims(), dtype=torch.bfloat16, device="cuda").normal_()
    torch.cuda.synchronize()
    return c


def _time_calls(eng, fn, reps, warm=2):
    """Median wall ms and stats of `fn` (which must end in kv_wait)."""
    ts, ko, ki = [], [], []
    for i in range(warm + reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn(i)
        dt = (time.perf_counter() - t0) * 1e3
        if i >= warm:
            st = eng.kv_last_stats()
            ts.append(dt); ko.append(st["ms_out"]); ki.append(st["ms_in"])
    return statistics.median(ts), statistics.median(ko), statistics.median(ki)


def _rot_calls(eng, rot):
    inv = rot.inverse()
    return (eng.prepare(rot.out_ids, rot.out_slots, rot.in_ids, rot.in_slots),
            eng.prepare(inv.out_ids, inv.out_slots, inv.in_ids, inv.in_slots))


def ladder(name="qwen25_32b"):
    """Naive -> per-block DMA -> one kernel per direction (serial) -> duplex, as in
    Table 2 of the paper (which ran 8 GB each way of Qwen2.5-32B KV on GH200)."""
    shape = W.SHAPES[name]
    link = B.kv_probe_link(256 << 20, 5)
    cache = _cache(shape)
    rot = W.config_rotation(name)
    inv = rot.inverse()
    blk = None
    rows = []

    def run(label, path, serial, reps, contiguous=False, layout=B.KV_HOST_BLOCK_FIRST):
        nonlocal blk
        r = W.config_rotation(name, contiguous_slots=contiguous)
        ri = r.inverse()
        eng = B.Engine(B.make_config(shape, layout, path), cache.data_ptr())
        blk = B.kv_block_bytes(eng.cfg)
        nbytes = len(r.out_ids) * blk
        if serial:
            t_out, t_in = [], []
            for i in range(reps + 1):
                a, b = (r, ri) if i % 2 == 0 else (ri, r)
                torch.cuda.synchronize(); t0 = time.perf_counter()
                assert eng.kv_swap_out(a.out_ids, a.out_slots) == 0 and eng.kv_wait() == 0
                t1 = time.perf_counter()
                assert eng.kv_swap_in(a.in_slots, a.in_ids) == 0 and eng.kv_wait() == 0
                t2 = time.perf_counter()
                if i >= 1:
                    t_out.append((t1 - t0) * 1e3); t_in.append((t2 - t1) * 1e3)
            mo, mi = statistics.median(t_out), statistics.median(t_in)
            rows.append((label, nbytes / mo / 1e6, "u", nbytes / mi / 1e6, "u", mo + mi))
        else:
            calls = _rot_calls(eng, r)

            def fn(i):
                assert calls[i & 1]() == 0 and eng.kv_wait() == 0
            ms, ko, ki = _time_calls(eng, fn, reps)
            rows.append((label, nbytes / ms / 1e6, "b", nbytes / ms / 1e6, "b", ms))
        eng.kv_destroy()
        print(f"  done: {label}", file=sys.stderr, flush=True)

    run("Naive: one hipMemcpyAsync per segment", B.KV_PATH_NAIVE, True, 1)
    run("MS analogue: pack kernel + one DMA copy per block", B.KV_PATH_SDMA_STAGED, True, 3)
    run("MS+MK analogue: one zero-copy kernel per direction, serial", B.KV_PATH_ZEROCOPY, True, 3)
    run("DMA staged, consecutive slots, both directions at once", B.KV_PATH_SDMA_STAGED, False, 3, contiguous=True)
    run("Two zero-copy kernels on two streams", B.KV_PATH_ZEROCOPY, False, 3)
    run("Fused duplex kernel (default)", B.KV_PATH_FUSED, False, 5)
    nbytes = len(rot.out_ids) * blk
    rows.append(("Ceiling: hipMemcpyAsync pinned, one way at a time", link["d2h"], "u", link["h2d"], "u",
                 nbytes / link["d2h"] / 1e6 + nbytes / link["h2d"] / 1e6))
    rows.append(("Ceiling: hipMemcpyAsync pinned, both ways at once", link["d2h_duplex"], "b",
                 link["h2d_duplex"], "b", nbytes / link["d2h_duplex"] / 1e6))
    print(f"\nLadder on {name}: {len(rot.out_ids)} blocks x {blk >> 20} MiB = {nbytes / 2**30:.1f} GiB per direction, "
          f"scattered block ids and slots\n")
    print("| Method | D2H GB/s | H2D GB/s | E2E ms |")
    print("|---|---|---|---|")
    for label, d, du, h, hu, ms in rows:
        print(f"| {label} | {d:.2f} ({du}) | {h:.2f} ({hu}) | {ms:.2f} |")


def layouts(name="qwen25_32b"):
    """Layer-first cache (this build's default) against the block-first cache the
    paper proposes, same workload as the ladder: rotation paths and the reader."""
    shape = W.SHAPES[name]
    cache = _cache(shape)
    rot = W.config_rotation(name)
    print(f"\n{name}: {len(rot.out_ids)} scattered blocks each way\n")
    print("| cache layout | method | D2H GB/s | H2D GB/s | E2E ms |")
    print("|---|---|---|---|---|")
    for hbm, hname in ((B.KV_HBM_LAYER_FIRST, "layer-first"), (B.KV_HBM_BLOCK_FIRST, "block-first")):
        plans = [("fused duplex kernel", B.KV_PATH_FUSED, False)]
        if hbm == B.KV_HBM_BLOCK_FIRST:
            plans += [("one DMA copy per block, one direction at a time (the paper's MS)", B.KV_PATH_DMA_BLOCKS, True),
                      ("one DMA copy per block, both directions at once", B.KV_PATH_DMA_BLOCKS, False)]
        else:
            plans += [("pack kernel + one DMA copy per block, one direction at a time", B.KV_PATH_SDMA_STAGED, True),
                      ("pack kernel + one DMA copy per block, both directions at once", B.KV_PATH_SDMA_STAGED, False)]
        for label, path, serial in plans:
            eng = B.Engine(B.make_config(shape, path=path, hbm_layout=hbm), cache.data_ptr())
            blk = B.kv_block_bytes(eng.cfg)
            nbytes = len(rot.out_ids) * blk
            inv = rot.inverse()
            if serial:
                to, ti = [], []
                for i in range(4):
                    a = rot if i % 2 == 0 else inv
                    torch.cuda.synchronize(); t0 = time.perf_counter()
                    assert eng.kv_swap_out(a.out_ids, a.out_slots) == 0 and eng.kv_wait() == 0
                    t1 = time.perf_counter()
                    assert eng.kv_swap_in(a.in_slots, a.in_ids) == 0 and eng.kv_wait() == 0
                    t2 = time.perf_counter()
                    if i:
                        to.append((t1 - t0) * 1e3); ti.append((t2 - t1) * 1e3)
                mo, mi = statistics.median(to), statistics.median(ti)
                print(f"| {hname} | {label} | {nbytes / mo / 1e6:.2f} (u) | {nbytes / mi / 1e6:.2f} (u) | {mo + mi:.2f} |", flush=True)
            else:
                calls = _rot_calls(eng, rot)

                def fn(i):
                    assert calls[i & 1]() == 0 and eng.kv_wait() == 0
                ms, _, _ = _time_calls(eng, fn, 4)
                print(f"| {hname} | {label} | {nbytes / ms / 1e6:.2f} (b) | {nbytes / ms / 1e6:.2f} (b) | {ms:.2f} |", flush=True)
            eng.kv_destroy()
    print("\n| cache layout | reader TB/s (all blocks of the cache, plane by plane) |")
    print("|---|---|")
    for hbm, hname in ((B.KV_HBM_LAYER_FIRST, "layer-first"), (B.KV_HBM_BLOCK_FIRST, "block-first")):
        eng = B.Engine(B.make_config(shape, hbm_layout=hbm), cache.data_ptr())
        blk = B.kv_block_bytes(eng.cfg)
        ids = np.random.default_rng(3).permutation(shape.n_hbm_blocks).astype(np.int32)
        assert eng.kv_reader_start(ids, 6) == 0
        rc, _, pm = eng.kv_reader_wait()
        print(f"| {hname} | {len(ids) * blk / statistics.median(pm[1:]) / 1e9:.2f} |", flush=True)
        eng.kv_destroy()


def linksweep():
    """Bandwidth against contiguous piece size, the analogue of the paper's link
    characterisation (Figs. 5 and 8): 256 MiB per direction moved as scattered
    segments of one size, by one DMA copy per segment and by the gather / scatter
    kernels; for the copies also the host time to enqueue one against the time
    the link needs for it."""
    print("\n| segment | copies per direction | per-copy DMA D2H GB/s | H2D GB/s | both ways at once GB/s (sum) | "
          "host us to enqueue a copy | device us per copy (one way) | link us / copy at 57 GB/s | kernel D2H GB/s (stores only) | "
          "kernel H2D GB/s (loads only) | fused both ways GB/s (sum) |")
    print("|---|---|---|---|---|---|---|---|---|---|---|")
    total = 256 << 20
    for seg in [4 << 10, 16 << 10, 32 << 10, 64 << 10, 256 << 10, 1 << 20, 4 << 20, 16 << 20, 64 << 20]:
        heads = seg // 4096                       # 16 tokens x heads x 128 dims x 2 bytes
        n = max(1, total // (2 * seg))            # one layer: a block is two segments
        n_copies = min(2 * n, 4096)
        n_naive = n_copies // 2
        nb = max(4 * n, 8)
        shape = W.KVShape(1, heads, 128, 16, n_hbm_blocks=nb, n_host_slots=2 * n + 2)
        cache = _cache(shape)
        rot = W.simple_rotation(shape, n, n, seed=seg)
        row = [f"{seg >> 10} KiB", str(2 * n_naive)]
        # one DMA copy per segment
        eng = B.Engine(B.make_config(shape, path=B.KV_PATH_NAIVE), cache.data_ptr())
        res = {}
        for d in ("out", "in", "both"):
            ts, enq = [], []
            for i in range(3):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                if d == "out":
                    assert eng.kv_swap_out(rot.out_ids[:n_naive], rot.out_slots[:n_naive]) == 0
                elif d == "in":
                    assert eng.kv_swap_in(rot.in_slots[:n_naive], rot.in_ids[:n_naive]) == 0
                else:
                    assert eng.kv_rotate(rot.out_ids[:n_naive], rot.out_slots[:n_naive], rot.in_ids[:n_naive],
                                         rot.in_slots[:n_naive]) == 0
                t1 = time.perf_counter()
                assert eng.kv_wait() == 0
                t2 = time.perf_counter()
                if i:
                    ts.append(t2 - t0); enq.append(t1 - t0)
            copies = 2 * n_naive * (2 if d == "both" else 1)
            # (GB/s, host us to enqueue one copy, wall us per copy)
            res[d] = (copies * seg / statistics.median(ts) / 1e9, statistics.median(enq) / copies * 1e6,
                      statistics.median(ts) / copies * 1e6)
        eng.kv_destroy()
        row += [f"{res['out'][0]:.2f}", f"{res['in'][0]:.2f}", f"{res['both'][0]:.2f}",
                f"{(res['out'][1] + res['in'][1]) / 2:.2f}", f"{(res['out'][2] + res['in'][2]) / 2:.2f}",
                f"{seg / 57e9 * 1e6:.2f}"]
        # gather / scatter kernels
        eng = B.Engine(B.make_config(shape), cache.data_ptr())
        inv = rot.inverse()
        for d in ("out", "in", "both"):
            ts = []
            for i in range(5):
                a = rot if i % 2 == 0 else inv
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                if d == "out":
                    rc = eng.kv_swap_out(a.out_ids, a.out_slots)
                elif d == "in":
                    rc = eng.kv_swap_in(a.in_slots, a.in_ids)
                else:
                    rc = eng.kv_rotate(a.out_ids, a.out_slots, a.in_ids, a.in_slots)
                assert rc == 0 and eng.kv_wait() == 0
                if i:
                    ts.append(time.perf_counter() - t0)
            moved = 2 * n * seg * (2 if d == "both" else 1)
            row.append(f"{moved / statistics.median(ts) / 1e9:.2f}")
        eng.kv_destroy()
        print("| " + " | ".join(row) + " |", flush=True)
        del cache
        torch.cuda.empty_cache()


def sizes():
    """Rotation rate against rotation size: n scattered blocks out while n come in
    (Llama-3-8B shape, 2 MiB blocks), one kv_rotate + kv_wait per step."""
    shape = W.SHAPES["llama3_8b"]
    cache = _cache(shape)
    eng = B.Engine(B.make_config(shape), cache.data_ptr())
    blk = B.kv_block_bytes(eng.cfg)
    print("\n| blocks each way | MiB each way | step us | out+in GB/s |")
    print("|---|---|---|---|")
    for n in [1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024]:
        rot = W.simple_rotation(shape, n, n, seed=n)
        calls = _rot_calls(eng, rot)

        def fn(i):
            assert calls[i & 1]() == 0 and eng.kv_wait() == 0
        ms, _, _ = _time_calls(eng, fn, 20 if n <= 128 else 6, warm=4)
        print(f"| {n} | {n * blk >> 20} | {ms * 1e3:.1f} | {2 * n * blk / ms / 1e6:.2f} |", flush=True)
    eng.kv_destroy()


def ratio():
    """The link's rate region as the engine sees it: one rotation with n_out : n_in
    scattered 2 MiB blocks (Llama-3-8B shape) at ratios from out-only to in-only."""
    shape = W.SHAPES["llama3_8b"]
    cache = _cache(shape)
    eng = B.Engine(B.make_config(shape), cache.data_ptr())
    blk = B.kv_block_bytes(eng.cfg)
    print("\n| out : in blocks | step ms | out GB/s | in GB/s | sum GB/s |")
    print("|---|---|---|---|---|")
    for n_out, n_in in [(1024, 0), (1024, 256), (1024, 512), (1024, 768), (1024, 896), (1024, 1024), (960, 1024),
                        (896, 1024), (832, 1024), (768, 1024), (512, 1024), (256, 1024), (0, 1024)]:
        rot = W.simple_rotation(shape, n_out, n_in, seed=n_out * 7 + n_in)
        calls = _rot_calls(eng, rot)
        # only the forward steps are timed; the inverse steps restore the state
        ts = []
        for i in range(12):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            assert calls[i & 1]() == 0 and eng.kv_wait() == 0
            if i >= 2 and not (i & 1):
                ts.append((time.perf_counter() - t0) * 1e3)
        ms = statistics.median(ts)
        print(f"| {n_out} : {n_in} | {ms:.2f} | {n_out * blk / ms / 1e6:.2f} | {n_in * blk / ms / 1e6:.2f} | "
              f"{(n_out + n_in) * blk / ms / 1e6:.2f} |", flush=True)
    eng.kv_destroy()


def chunks(name="long70b"):
    """What the chunk pipeline of the DMA-staged path costs.  Chunks of one
    direction run strictly one after the other on that direction's stream (pack,
    copies, pack, ...), so every chunk adds its pack (or unpack) kernel and the
    kernel <-> copy hand-overs to the direction's time.  The same 20 + 20 GiB
    rotation with chunks from 64 MiB to 1 GiB: step time against the number of
    chunks gives that cost per chunk, i.e. what double-buffered overlap could
    win back; the DMA engines' own both-ways rate is the ceiling of the path."""
    shape = W.SHAPES[name]
    link = B.kv_probe_link(1 << 30, 5)
    print(f"\nhipMemcpyAsync pinned, 1 GiB: D2H {link['d2h']:.2f}, H2D {link['h2d']:.2f}, both at once "
          f"{link['d2h_duplex']:.2f} GB/s per direction (the DMA engines' ceiling for this path)\n")
    cache = _cache(shape)
    rot = W.config_rotation(name, contiguous_slots=True)
    print("| path | chunk MiB | chunks per direction | kernels + copies | step ms | GB/s per direction | "
          "of the DMA both-ways ceiling |")
    print("|---|---|---|---|---|---|---|")
    plane_pair = 2 * len(rot.out_ids) * B.kv_seg_bytes(B.make_config(shape))     # one layer of the whole list
    rows = []
    plans = [(1, plane_pair // 4), (1, plane_pair // 2), (1, plane_pair), (2, 2 * plane_pair), (4, 4 * plane_pair)]
    for chunk_layers, staging in plans:
        eng = B.Engine(B.make_config(shape, B.KV_HOST_LAYER_FIRST, B.KV_PATH_SDMA_STAGED, chunk_layers=chunk_layers,
                                     staging_bytes=staging), cache.data_ptr())
        blk = B.kv_block_bytes(eng.cfg)
        calls = _rot_calls(eng, rot)

        def fn(i):
            assert calls[i & 1]() == 0 and eng.kv_wait() == 0
        ms, _, _ = _time_calls(eng, fn, 4, warm=2)
        st = eng.kv_last_stats()
        n_chunks = len(rot.out_ids) * blk // staging
        gbps = len(rot.out_ids) * blk / ms / 1e6
        rows.append((n_chunks, ms))
        print(f"| DMA staged, layer-first pool, consecutive slots | {staging >> 20} | {n_chunks} | {st['n_launches']} | "
              f"{ms:.1f} | {gbps:.2f} | {100 * gbps / link['d2h_duplex']:.1f} % |", flush=True)
        eng.kv_destroy()
    eng = B.Engine(B.make_config(shape), cache.data_ptr())
    blk = B.kv_block_bytes(eng.cfg)
    calls = _rot_calls(eng, W.config_rotation(name))

    def fn(i):
        assert calls[i & 1]() == 0 and eng.kv_wait() == 0
    ms, _, _ = _time_calls(eng, fn, 4, warm=2)
    gbps = len(rot.out_ids) * blk / ms / 1e6
    print(f"| fused kernel, scattered slots (default) | - | - | {eng.kv_last_stats()['n_launches']} | {ms:.1f} | "
          f"{gbps:.2f} | {100 * gbps / link['d2h_duplex']:.1f} % |", flush=True)
    eng.kv_destroy()
    # least squares: step ms = a + b * chunks
    xs, ys = [r[0] for r in rows], [r[1] for r in rows]
    mx, my = sum(xs) / len(xs), sum(ys) / len(ys)
    b = sum((x - mx) * (y - my) for x, y in zip(xs, ys)) / sum((x - mx) ** 2 for x in xs)
    a = my - b * mx
    print(f"\nfit: step ms = {a:.1f} + {b * 1e3:.1f} us x chunks per direction; with one chunk per layer "
          f"(80 chunks) the serial hand-overs cost {80 * b:.1f} ms = {100 * 80 * b / (a + 80 * b):.1f} % of the step")


def layers(name="long70b"):
    """The default path layer by layer (cfg.chunk_layers > 0): one launch per chunk
    of layers with a completion mark each, so that a consumer can start on layer l
    while later layers move.  For configs[3] (20 + 20 GiB, 80 layers): what the
    chunks cost the whole rotation, and when the first and the middle layer are
    in place (host clock from the call, kv_wait_layer)."""
    shape = W.SHAPES[name]
    cache = _cache(shape)
    rot = W.config_rotation(name)
    print(f"\n{name}: {len(rot.out_ids)} blocks out while {len(rot.in_ids)} come in, "
          f"{len(rot.out_ids) * B.kv_block_bytes(B.make_config(shape)) / 2**30:.0f} GiB each way, {shape.n_layers} layers\n")
    print("| layers per launch | launches | MiB per launch and direction | whole rotation ms | GB/s per direction | "
          "layer 0 in place after ms | middle layer in place after ms |")
    print("|---|---|---|---|---|---|---|")
    for chunk in (0, 16, 8, 4, 2, 1):
        eng = B.Engine(B.make_config(shape, chunk_layers=chunk), cache.data_ptr())
        blk = B.kv_block_bytes(eng.cfg)
        calls = _rot_calls(eng, rot)
        t_all, t_first, t_mid = [], [], []
        for i in range(6):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            assert calls[i & 1]() == 0
            assert eng.kv_wait_layer(0) == 0
            t1 = time.perf_counter()
            assert eng.kv_wait_layer(shape.n_layers // 2) == 0
            t2 = time.perf_counter()
            assert eng.kv_wait() == 0
            t3 = time.perf_counter()
            if i >= 2:
                t_first.append((t1 - t0) * 1e3); t_mid.append((t2 - t0) * 1e3); t_all.append((t3 - t0) * 1e3)
        ms = statistics.median(t_all)
        n_launch = eng.kv_last_stats()["n_launches"]
        per = len(rot.out_ids) * blk / n_launch / 2**20
        print(f"| {chunk if chunk else 'all (one launch)'} | {n_launch} | {per:.0f} | {ms:.1f} | "
              f"{len(rot.out_ids) * blk / ms / 1e6:.2f} | {statistics.median(t_first):.1f} | {statistics.median(t_mid):.1f} |",
              flush=True)
        eng.kv_destroy()


def poolkinds():
    """The pool as different kinds of pinned host memory (hipHostMalloc flags),
    handed to the engine as a caller-owned pool: the configs[1] rotation, a
    2 + 2 GiB rotation and each direction alone."""
    import ctypes as C
    hip = C.CDLL("libamdhip64.so")      # the runtime torch has already loaded
    hip.hipHostMalloc.argtypes = [C.POINTER(C.c_void_p), C.c_size_t, C.c_uint]
    hip.hipHostFree.argtypes = [C.c_void_p]
    shape = W.SHAPES["llama3_8b"]
    cache = _cache(shape)
    rot, big = W.config_rotation("llama3_8b"), W.simple_rotation(shape, 1024, 1024, seed=3)
    kinds = [("default (what the engine allocates)", 0), ("portable + mapped", 0x3), ("write-combined", 0x4),
             ("coherent", 0x40000000), ("non-coherent", 0x80000000), ("non-coherent + write-combined", 0x80000004),
             ("NUMA-user", 0x20000000)]
    print("\n| hipHostMalloc flags | 128 + 128 blocks GB/s (sum) | 1024 + 1024 blocks GB/s (sum) | swap-out alone GB/s | swap-in alone GB/s |")
    print("|---|---|---|---|---|")
    for name, flags in kinds:
        cfg = B.make_config(shape)
        blk = B.kv_block_bytes(cfg)
        ptr = C.c_void_p()
        if hip.hipHostMalloc(C.byref(ptr), B.kv_pool_bytes(cfg), flags) != 0:
            print(f"| {name} | allocation refused | | | |", flush=True)
            continue
        eng = B.Engine(cfg, cache.data_ptr(), ptr.value)
        row = []
        for r in (rot, big):
            calls = _rot_calls(eng, r)

            def fn(i):
                assert calls[i & 1]() == 0 and eng.kv_wait() == 0
            ms, _, _ = _time_calls(eng, fn, 20, warm=4)
            row.append((len(r.out_ids) + len(r.in_ids)) * blk / ms / 1e6)

        def out_only(i):
            assert eng.kv_swap_out(big.out_ids, big.out_slots) == 0 and eng.kv_wait() == 0

        def in_only(i):
            assert eng.kv_swap_in(big.out_slots, big.out_ids) == 0 and eng.kv_wait() == 0
        for fn in (out_only, in_only):
            ms, _, _ = _time_calls(eng, fn, 10, warm=2)
            row.append(len(big.out_ids) * blk / ms / 1e6)
        print(f"| {name} | " + " | ".join(f"{v:.2f}" for v in row) + " |", flush=True)
        eng.kv_destroy()
        hip.hipHostFree(ptr)


def splitcalls():
    """configs[2] (32 requests out, 32 in, lognormal lengths) moved (a) in one call,
    (b) as 32 calls of one request pair each with a kv_wait after every call,
    (c) as the same 32 calls enqueued back to back with one kv_wait at the end.
    (b) holds each call's own imbalance (|out_i - in_i| runs at the one-way rate)
    and 32 launch-and-wait round trips; what (c) has beyond (b) minus those round
    trips is lost between launches."""
    shape = W.SHAPES["batch"]
    cache = _cache(shape)
    info = W.batch_rotation(shape, W.BASE_SEED + 102)
    rot = info["rotation"]; bo_, bi_ = info["bounds_out"], info["bounds_in"]
    inv = rot.inverse()
    eng = B.Engine(B.make_config(shape), cache.data_ptr())
    blk = B.kv_block_bytes(eng.cfg)
    whole = _rot_calls(eng, rot)
    pairs_f, pairs_b, sizes_ = [], [], []
    for r in range(len(bo_) - 1):
        o, i_ = slice(bo_[r], bo_[r + 1]), slice(bi_[r], bi_[r + 1])
        pairs_f.append(eng.prepare(rot.out_ids[o], rot.out_slots[o], rot.in_ids[i_], rot.in_slots[i_]))
        pairs_b.append(eng.prepare(inv.out_ids[i_], inv.out_slots[i_], inv.in_ids[o], inv.in_slots[o]))
        sizes_.append((bo_[r + 1] - bo_[r], bi_[r + 1] - bi_[r]))

    def timed(fn_f, fn_b, reps=8):
        f, b = [], []
        for i in range(2 + reps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            (fn_b if i & 1 else fn_f)()
            if i >= 2:
                (b if i & 1 else f).append((time.perf_counter() - t0) * 1e3)
        return statistics.median(f), statistics.median(b)

    def one(c):
        def go():
            assert c() == 0 and eng.kv_wait() == 0
        return go

    def each_waited(cs):
        def go():
            for c in cs:
                assert c() == 0 and eng.kv_wait() == 0
        return go

    def unwaited(cs):
        def go():
            for c in cs:
                assert c() == 0
            assert eng.kv_wait() == 0
        return go

    a = timed(one(whole[0]), one(whole[1]))
    b = timed(each_waited(pairs_f), each_waited(pairs_b))
    c = timed(unwaited(pairs_f), unwaited(pairs_b))
    # launch-and-wait round trip of a call that moves one block each way
    tiny = W.simple_rotation(shape, 1, 1, seed=9)
    tc = _rot_calls(eng, tiny)
    t1 = timed(one(tc[0]), one(tc[1]), reps=40)
    fixed_ms = min(t1) - 2 * blk / 100.7e6
    so = sum(abs(o - i) for o, i in sizes_)
    print(f"\n{len(rot.out_ids)} blocks out, {len(rot.in_ids)} in; sum over the 32 pairs of |out_i - in_i| = {so} blocks "
          f"against |sum out - sum in| = {abs(len(rot.out_ids) - len(rot.in_ids))}; a call that moves one block each "
          f"way and waits takes {min(t1) * 1e3:.0f} us, of which {fixed_ms * 1e3:.0f} us are not link time\n")
    print("| how | forward ms (out-heavy) | inverse ms (in-heavy) | launches |")
    print("|---|---|---|---|")
    print(f"| one call | {a[0]:.2f} | {a[1]:.2f} | 2 / 1 |")
    print(f"| 32 calls, each waited for | {b[0]:.2f} | {b[1]:.2f} | |")
    print(f"| 32 calls back to back, one wait | {c[0]:.2f} | {c[1]:.2f} | {eng.kv_last_stats()['n_launches']} |")
    print(f"| (each waited) - 32 round trips | {b[0] - 32 * fixed_ms:.2f} | {b[1] - 32 * fixed_ms:.2f} | |")
    print(f"\nlost between launches, back to back: forward {c[0] - (b[0] - 32 * fixed_ms):+.2f} ms, inverse "
          f"{c[1] - (b[1] - 32 * fixed_ms):+.2f} ms; lost to per-call imbalance: forward "
          f"{b[0] - 32 * fixed_ms - a[0]:+.2f} ms, inverse {b[1] - 32 * fixed_ms - a[1]:+.2f} ms", flush=True)
    eng.kv_destroy()


def packalone(name="llama3_8b"):
    """Pack and unpack kernels of the DMA-staged path with nothing running beside
    them: swap-outs and swap-ins of configs[1]'s 128 blocks in turn, each waited
    for.  Meant to run under rocprofv3 --kernel-trace --stats, which gives the
    kernel durations (both directions at once would put the other direction's
    copies beside each kernel, and under the profiler those copies are kernels)."""
    shape = W.SHAPES[name]
    cache = _cache(shape)
    rot = W.config_rotation(name, contiguous_slots=True)
    eng = B.Engine(B.make_config(shape, path=B.KV_PATH_SDMA_STAGED), cache.data_ptr())
    blk = B.kv_block_bytes(eng.cfg)
    to, ti = [], []
    for i in range(44):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if i % 2 == 0:
            assert eng.kv_swap_out(rot.out_ids, rot.out_slots) == 0
        else:
            assert eng.kv_swap_in(rot.out_slots, rot.out_ids) == 0
        assert eng.kv_wait() == 0
        if i >= 4:
            (ti if i % 2 else to).append((time.perf_counter() - t0) * 1e3)
    # a plain 256 MiB device copy of known size, the reference for scaling the profiler's
    # FETCH_SIZE / WRITE_SIZE readings
    a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_()
    b = torch.empty_like(a)
    for _ in range(3):
        b.copy_(a)
    torch.cuda.synchronize()
    mb = len(rot.out_ids) * blk
    print(f"swap-out alone (pack + one DMA copy, {mb >> 20} MiB): {statistics.median(to):.3f} ms = "
          f"{mb / statistics.median(to) / 1e6:.2f} GB/s; swap-in alone (one DMA copy + unpack): "
          f"{statistics.median(ti):.3f} ms = {mb / statistics.median(ti) / 1e6:.2f} GB/s", flush=True)
    eng.kv_destroy()


def packshapes():
    """Runs the stand-alone measurement program csrc/pack_probe.hip (built by
    paper_2601_20309_amd.build.build_probe) and passes its table through."""
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "pack_probe")
    if not os.path.exists(exe):
        sys.exit(f"{exe} is not built: run python -c 'from paper_2601_20309_amd import build; build.build_probe()'")
    raise SystemExit(subprocess.run([exe]).returncode)


def configs():
    link = B.kv_probe_link(256 << 20, 5)
    print(f"\nhipMemcpyAsync pinned peaks: D2H {link['d2h']:.2f}, H2D {link['h2d']:.2f}, both at once "
          f"{link['d2h_duplex']:.2f} per direction (GB/s)\n")
    print("| Config | path | out GiB | in GiB | step ms | out GB/s | in GB/s | % of D2H peak | % of H2D peak | launches |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    plans = [
        ("llama3_8b", dict(), "default"),
        ("llama3_8b", dict(host_layout=B.KV_HOST_LAYER_FIRST), "layer-first pool"),
        ("batch", dict(), "default"),
        ("long70b", dict(), "default (one launch)"),
        ("long70b", dict(path=B.KV_PATH_SDMA_STAGED, host_layout=B.KV_HOST_LAYER_FIRST, chunk_layers=1,
                         staging_bytes=512 << 20), "DMA staged, per-layer chunks, consecutive slots"),
    ]
    cache, cache_name = None, None
    for name, kw, label in plans:
        shape = W.SHAPES[name]
        if cache_name != (shape.cache_dims()):
            del cache
            torch.cuda.empty_cache()
            cache, cache_name = _cache(shape), shape.cache_dims()
        contiguous = kw.get("path") == B.KV_PATH_SDMA_STAGED
        rot = W.config_rotation(name, contiguous_slots=contiguous)
        eng = B.Engine(B.make_config(shape, **kw), cache.data_ptr())
        blk = B.kv_block_bytes(eng.cfg)
        calls = _rot_calls(eng, rot)

        # forward and inverse steps alternate (state returns); an unbalanced rotation is
        # out-heavy one way and in-heavy the other, so the two are timed apart
        fwd, bwd = [], []
        for i in range(2 + 2 * (6 if name == "llama3_8b" else 4)):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            assert calls[i & 1]() == 0 and eng.kv_wait() == 0
            if i >= 2:
                (bwd if i & 1 else fwd).append((time.perf_counter() - t0) * 1e3)
        st = eng.kv_last_stats()
        bo, bi = len(rot.out_ids) * blk, len(rot.in_ids) * blk
        rows = [(label, statistics.median(fwd + bwd), bo, bi)] if bo == bi else \
            [(label, statistics.median(fwd), bo, bi), (label + ", the inverse rotation", statistics.median(bwd), bi, bo)]
        for lab, ms, b_out, b_in in rows:
            go, gi = b_out / ms / 1e6, b_in / ms / 1e6
            print(f"| {name} | {lab} ({B.PATH_NAMES[st['path_used']]}) | {b_out / 2**30:.2f} | {b_in / 2**30:.2f} | "
                  f"{ms:.3f} | {go:.2f} | {gi:.2f} | {100 * go / link['d2h']:.1f} | {100 * gi / link['h2d']:.1f} | "
                  f"{st['n_launches']} |", flush=True)
        eng.kv_destroy()
    # configs[2] again as 32 back-to-back calls, one request pair each
    shape = W.SHAPES["batch"]
    del cache
    torch.cuda.empty_cache()
    cache = _cache(shape)
    info = W.batch_rotation(shape, W.BASE_SEED + 102)
    rot = info["rotation"]; bo_, bi_ = info["bounds_out"], info["bounds_in"]
    eng = B.Engine(B.make_config(shape), cache.data_ptr())
    blk = B.kv_block_bytes(eng.cfg)
    pairs_f, pairs_b = [], []
    inv = rot.inverse()
    for r in range(len(bo_) - 1):
        o, i_ = slice(bo_[r], bo_[r + 1]), slice(bi_[r], bi_[r + 1])
        pairs_f.append(eng.prepare(rot.out_ids[o], rot.out_slots[o], rot.in_ids[i_], rot.in_slots[i_]))
        pairs_b.append(eng.prepare(inv.out_ids[i_], inv.out_slots[i_], inv.in_ids[o], inv.in_slots[o]))

    fwd, bwd = [], []
    for i in range(10):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for c in (pairs_f if i % 2 == 0 else pairs_b):
            assert c() == 0
        assert eng.kv_wait() == 0
        if i >= 2:
            (bwd if i & 1 else fwd).append((time.perf_counter() - t0) * 1e3)
    bo, bi = len(rot.out_ids) * blk, len(rot.in_ids) * blk
    for lab, ms, b_out, b_in in [("", statistics.median(fwd), bo, bi),
                                 (", the inverse rotations", statistics.median(bwd), bi, bo)]:
        print(f"| batch | default, {len(pairs_f)} calls of one request pair each, one kv_wait{lab} | {b_out / 2**30:.2f} | "
              f"{b_in / 2**30:.2f} | {ms:.3f} | {b_out / ms / 1e6:.2f} | {b_in / ms / 1e6:.2f} | "
              f"{100 * b_out / ms / 1e6 / link['d2h']:.1f} | {100 * b_in / ms / 1e6 / link['h2d']:.1f} | "
              f"{eng.kv_last_stats()['n_launches']} |")
    eng.kv_destroy()


def interference():
    """configs[4]: 8 x 4096-token requests each way while a reader streams the KV
    of 19200 other blocks (37.5 GiB) layer by layer."""
    name = "interference"
    shape = W.SHAPES[name]
    link = B.kv_probe_link(256 << 20, 5)
    cache = _cache(shape)
    print(f"\nhipMemcpyAsync pinned peaks: D2H {link['d2h']:.2f}, H2D {link['h2d']:.2f} GB/s\n")
    print("| rotation path | copy WGs x lanes | rotation alone GB/s (out+in) | rotation beside reader GB/s | "
          "reader alone TB/s | reader beside rotation TB/s | reader time lost, ms per GiB moved |")
    print("|---|---|---|---|---|---|---|")
    for path, wgs, lanes, contiguous in [(B.KV_PATH_FUSED, 0, 0, False), (B.KV_PATH_FUSED, 192, 64, False),
                                         (B.KV_PATH_FUSED, 144, 64, False), (B.KV_PATH_FUSED, 96, 64, False),
                                         (B.KV_PATH_FUSED, 80, 64, False), (B.KV_PATH_FUSED, 64, 64, False),
                                         (B.KV_PATH_FUSED, 28, 256, False), (B.KV_PATH_FUSED, 16, 448, False),
                                         (B.KV_PATH_FUSED, 8, 896, False),
                                         (B.KV_PATH_SDMA_STAGED, 0, 0, True), (B.KV_PATH_DMA_BLOCKS, 0, 0, False)]:
        rot = W.config_rotation(name, contiguous_slots=contiguous)
        named = np.zeros(shape.n_hbm_blocks, bool)
        named[rot.out_ids] = True; named[rot.in_ids] = True
        others = np.flatnonzero(~named)[:19200].astype(np.int32)
        # one DMA copy per block needs whole blocks to be contiguous: the block-first cache
        hbm_layout = B.KV_HBM_BLOCK_FIRST if path == B.KV_PATH_DMA_BLOCKS else B.KV_HBM_LAYER_FIRST
        eng = B.Engine(B.make_config(shape, path=path, max_copy_wgs=wgs, wg_lanes=lanes, hbm_layout=hbm_layout),
                       cache.data_ptr())
        blk = B.kv_block_bytes(eng.cfg)
        calls = _rot_calls(eng, rot)
        moved = (len(rot.out_ids) + len(rot.in_ids)) * blk
        read_bytes = len(others) * blk

        def alone(i):
            assert calls[i & 1]() == 0 and eng.kv_wait() == 0
        ms_alone, _, _ = _time_calls(eng, alone, 4)
        # reader alone
        assert eng.kv_reader_start(others, 6) == 0
        rc, _, pm = eng.kv_reader_wait()
        read_alone = read_bytes / statistics.median(pm[1:]) / 1e9
        # both: enough reader passes to outlast the rotation
        n_pass = min(256, int(ms_alone / statistics.median(pm[1:]) * 1.5) + 4)
        both = []
        read_both = []
        for i in range(4):
            torch.cuda.synchronize()
            assert eng.kv_reader_start(others, n_pass) == 0
            t0 = time.perf_counter()
            assert calls[i & 1]() == 0 and eng.kv_wait() == 0
            dt = (time.perf_counter() - t0) * 1e3
            rc, _, pm2 = eng.kv_reader_wait()
            assert rc == 0
            if i >= 1:
                both.append(dt)
                # passes that ran entirely inside the rotation window: bytes read / their time
                acc, inside = 0.0, []
                for p in pm2:
                    if acc + p <= dt:
                        inside.append(p)
                    acc += p
                inside = inside[1:] or pm2      # the first one started before the rotation
                read_both.append(read_bytes * len(inside) / sum(inside) / 1e9)
        ms_both = statistics.median(both)
        launch = ("no kernel, block-first cache" if path == B.KV_PATH_DMA_BLOCKS else "pack / unpack kernels"
                  if path != B.KV_PATH_FUSED else f"{wgs} x {lanes}" if wgs else "default (112 x 64)")
        # what the co-runner pays: the part of the rotation's duration in which it got nothing done
        rb = statistics.median(read_both)
        lost = ms_both * (1 - rb / read_alone) / (moved / 2**30)
        print(f"| {B.PATH_NAMES[path]} | {launch} | {moved / ms_alone / 1e6:.2f} | {moved / ms_both / 1e6:.2f} | "
              f"{read_alone:.2f} | {rb:.2f} | {lost:.2f} |", flush=True)
        eng.kv_destroy()
    # one direction at a time (what the eager step and a plain resumption issue), default shapes
    print("\n| one direction, default shape | alone GB/s | beside reader GB/s | reader alone TB/s | reader beside TB/s | "
          "reader time lost, ms per GiB moved |")
    print("|---|---|---|---|---|---|")
    rot = W.config_rotation(name, contiguous_slots=False)
    inv = rot.inverse()
    named = np.zeros(shape.n_hbm_blocks, bool)
    named[rot.out_ids] = True; named[rot.in_ids] = True
    others = np.flatnonzero(~named)[:19200].astype(np.int32)
    eng = B.Engine(B.make_config(shape), cache.data_ptr())
    blk = B.kv_block_bytes(eng.cfg)
    read_bytes = len(others) * blk
    assert eng.kv_reader_start(others, 6) == 0
    rc, _, pm = eng.kv_reader_wait()
    ms_pass = statistics.median(pm[1:])
    for d, label in (("out", "swap-out (12 waves x 8 vectors)"), ("in", "swap-in (24 waves x 4 vectors)")):
        def one(i):
            a = rot if i % 2 == 0 else inv
            rc = eng.kv_swap_out(a.out_ids, a.out_slots) if d == "out" else eng.kv_swap_in(a.in_slots, a.in_ids)
            assert rc == 0 and eng.kv_wait() == 0
        n_moved = (len(rot.out_ids) if d == "out" else len(rot.in_ids)) * blk
        ms_alone, _, _ = _time_calls(eng, one, 4)
        both, read_both = [], []
        for i in range(4):
            torch.cuda.synchronize()
            assert eng.kv_reader_start(others, min(256, int(ms_alone / ms_pass * 1.5) + 4)) == 0
            t0 = time.perf_counter()
            one(i)
            dt = (time.perf_counter() - t0) * 1e3
            rc, _, pm2 = eng.kv_reader_wait()
            assert rc == 0
            if i >= 1:
                both.append(dt)
                acc, inside = 0.0, []
                for p in pm2:
                    if acc + p <= dt:
                        inside.append(p)
                    acc += p
                inside = inside[1:] or pm2
                read_both.append(read_bytes * len(inside) / sum(inside) / 1e9)
        rb, ra = statistics.median(read_both), read_bytes / ms_pass / 1e9
        lost = statistics.median(both) * (1 - rb / ra) / (n_moved / 2**30)
        print(f"| {label} | {n_moved / ms_alone / 1e6:.2f} | {n_moved / statistics.median(both) / 1e6:.2f} | "
              f"{ra:.2f} | {rb:.2f} | {lost:.2f} |", flush=True)
    eng.kv_destroy()


def reader():
    """The decode reader alone (for profiling): 8 passes over 19200 blocks, plus a
    plain 256 MiB device copy as the known-size reference for the counters."""
    shape = W.SHAPES["interference"]
    cache = _cache(shape)
    eng = B.Engine(B.make_config(shape), cache.data_ptr())
    blk = B.kv_block_bytes(eng.cfg)
    ids = np.arange(19200, dtype=np.int32)
    a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_()
    b = torch.empty_like(a)
    for _ in range(3):
        b.copy_(a)
    torch.cuda.synchronize()
    assert eng.kv_reader_start(ids, 8) == 0
    rc, _, pm = eng.kv_reader_wait()
    assert rc == 0
    ms = statistics.median(pm[1:])
    nbytes = len(ids) * blk
    print(f"kv_reader_kernel: {nbytes / 2**30:.2f} GiB per pass, median pass {ms:.3f} ms = {nbytes / ms / 1e9:.3f} TB/s "
          f"= {100 * nbytes / ms / 1e9 / 8.0:.1f} % of the 8 TB/s HBM peak")
    eng.kv_destroy()


def eager():
    """What eager block rotation buys at a preemption (Section 4.3.2): 8 requests
    of 4096 tokens leave while 8 others come back, Llama-3-8B shape, with and
    without the background copies having been issued beforehand; and what the
    eager copies of 6 further requests cost when they ride in that rotation."""
    base = W.SHAPES["interference"]
    shape = W.KVShape(base.n_layers, base.n_kv_heads, base.head_dim, base.block_size,
                      n_hbm_blocks=base.n_hbm_blocks, n_host_slots=8192)
    cache = _cache(shape)
    print("\n| eager step before the rotation | blocks copied out at preemption | dropped without a copy | "
          "eager copies riding along | blocks swapped in | rotation ms | out GiB | in GiB |")
    print("|---|---|---|---|---|---|---|---|")
    for do_eager, ride in ((False, 0), (True, 0), (True, 1536)):
        eng = B.Engine(B.make_config(shape), cache.data_ptr())
        tab = B.Table(eng, 32)
        for r in range(16):
            assert tab.kv_table_append(r, 4096 - 5)[0] == 0      # 255 full blocks + a dirty tail
        assert tab.kv_table_rotate(list(range(8, 16)), []) == 0   # 8 requests wait in DRAM
        assert eng.kv_wait() == 0
        t_eager = 0.0
        if do_eager:
            t0 = time.perf_counter()
            rc, n = tab.kv_table_eager(1 << 30)
            assert rc == 0 and eng.kv_wait() == 0
            t_eager = (time.perf_counter() - t0) * 1e3
        for r in range(16, 22 if ride else 16):
            assert tab.kv_table_append(r, 4096)[0] == 0           # 256 full blocks each, not yet copied
        c0 = tab.kv_table_get_counts()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rc, n_ride = tab.kv_table_rotate_eager(list(range(8)), list(range(8, 16)), ride)
        assert rc == 0 and n_ride == ride and eng.kv_wait() == 0
        ms = (time.perf_counter() - t0) * 1e3
        c1 = tab.kv_table_get_counts()
        st = eng.kv_last_stats()
        label = f"yes ({n} blocks, {t_eager:.1f} ms in the background)" if do_eager else "no"
        print(f"| {label} | {c1['copied_preempt'] - c0['copied_preempt']} | {c1['dropped_synced'] - c0['dropped_synced']} | "
              f"{n_ride} | {c1['swapped_in'] - c0['swapped_in']} | {ms:.2f} | {st['bytes_out'] / 2**30:.3f} | "
              f"{st['bytes_in'] / 2**30:.3f} |", flush=True)
        tab.kv_table_destroy()
        eng.kv_destroy()


def fit_picks(pre, pri, state, blocks_of, free_hbm, b_xfer, headroom):
    """Harness policy of the serving loops (not part of the method): which of the
    requests LVF prioritised really start this iteration.  `room` is what the
    cache holds once the preempted have left, minus `headroom` blocks kept for
    the tokens the running batch is about to append; a request needs its blocks
    plus one to grow into; a rotary request also needs its blocks in swap-in
    budget, since B_xfer bounds what one iteration swaps (Section 4.2.2).  A
    request that does not fit is skipped and stays where it is.
    Returns (admit, resume): waiting requests to prefill, rotary ones to swap in."""
    admit, resume = [], []
    room = free_hbm + sum(blocks_of(r) for r in pre) - headroom
    swap_in_left = b_xfer
    for r in pri:
        need = blocks_of(r) + 1
        if need > room:
            continue
        if state[r] == B.KV_REQ_ROTARY:
            if need - 1 > swap_in_left:
                continue
            swap_in_left -= need - 1
            resume.append(r)
        else:
            admit.append(r)
        room -= need
    return admit, resume


def serve(rps=45.0, seconds=20.0, seed=0, b_xfer=None, hbm_blocks=4096, host_slots=16384, exec_passes=1):
    """Cross-iteration pipeline (Section 4.3.2) with synthetic traffic.  Iteration t
    "executes" on the GPU (the decode reader streams a weights-sized read on its
    own stream) while the host prepares iteration t+1: LVF (Algorithm 1) picks
    what rotates and the block table enqueues the transfer, eager copies
    included.  An iteration stalls when its preparation (scheduling + transfer,
    on the host clock from the start of the execution) outlasts the execution:
    the quantities of the paper's Section 5.4 stall paragraph.  exec_passes: how
    many times the reader goes over its 16 GiB per iteration (1: ~2.5 ms; 28: ~70 ms,
    the execution time the paper reports)."""
    shape = W.SHAPES["llama3_8b"]                 # blocks of 16 tokens; a small cache so that requests must rotate
    shape = W.KVShape(shape.n_layers, shape.n_kv_heads, shape.head_dim, shape.block_size,
                      n_hbm_blocks=hbm_blocks, n_host_slots=host_slots)
    P = shape.block_size
    cache = _cache(shape)
    eng = B.Engine(B.make_config(shape), cache.data_ptr())
    tab = B.Table(eng, 4096)
    blk = B.kv_block_bytes(eng.cfg)
    params = (3.0, 0.0, 0.5, 0.1, 5.0)            # alpha, beta_B, beta_F, S_B = 100 ms, S_F = 5 s (Section 5.1)
    rng = np.random.default_rng(seed)
    # a 16 GiB read per iteration stands for the model weights (Llama-3-8B in bf16)
    # (the batch's own KV lies inside it: the reader takes at most 2 x hbm_blocks ids)
    weights_ids = (np.arange(0, min(8192, 2 * hbm_blocks), dtype=np.int64) % hbm_blocks).astype(np.int32)
    # link budget per iteration: what 80 % of the measured both-ways rate moves during one
    # execution, re-derived from the running average of the execution time
    fixed_budget = b_xfer
    b_xfer = fixed_budget if fixed_budget is not None else int(0.8 * 48e9 * 2.6e-3 * exec_passes / blk)
    arrivals = np.cumsum(rng.exponential(1.0 / rps, size=int(rps * seconds * 1.2) + 8))
    prompts = np.clip(np.rint(rng.lognormal(np.log(700), 0.9, size=arrivals.size)), 16, 8192).astype(int)
    outputs = np.clip(np.rint(rng.lognormal(np.log(200), 0.8, size=arrivals.size)), 4, 2048).astype(int)
    state, t_ref, length, target = {}, {}, {}, {}
    ttft, tbt, first_done = [], [], set()
    free_ids = list(range(4095, -1, -1))
    now, next_arrival, it = 0.0, 0, 0
    n_stall, n_rot, t_sched, t_xfer, t_prep, t_exec, moved_blocks = 0, 0, [], [], [], [], 0
    arrive_time = {}
    blocks_of = lambda r: -(-length[r] // P)
    while now < seconds:
        while next_arrival < arrivals.size and arrivals[next_arrival] <= now and free_ids:
            r = free_ids.pop()
            state[r], t_ref[r] = B.KV_REQ_WAITING, float(arrivals[next_arrival])
            arrive_time[r] = float(arrivals[next_arrival])
            length[r], target[r] = int(prompts[next_arrival]), int(prompts[next_arrival] + outputs[next_arrival])
            next_arrival += 1
        # ---- GPU: iteration t executes ---------------------------------------------------------------
        batch = [r for r in state if state[r] == B.KV_REQ_RUNNING]
        x0 = time.perf_counter()
        assert eng.kv_reader_start(weights_ids, exec_passes) == 0
        # ---- host, meanwhile: schedule iteration t+1 and enqueue its rotation --------------------------
        h0 = time.perf_counter()
        reqs = [(r, state[r], blocks_of(r), t_ref[r]) for r in state]
        free_hbm = tab.kv_table_get_counts()["free_hbm_blocks"]
        rc, pre, pri, fcfs = B.kv_sched_lvf(params, reqs, now, b_xfer, free_hbm)
        assert rc == 0
        running_after = [r for r in batch if r not in pre]
        admit, resume = fit_picks(pre, pri, state, blocks_of, free_hbm, b_xfer, headroom=len(running_after) + 8)
        # the eager step rides in the rotation's transfer: swap-out bytes up to ~0.8 x the
        # swap-in bytes cost no link time
        spent = sum(blocks_of(r) for r in resume) + len(pre)
        rc, n_eager = tab.kv_table_rotate_eager(pre, resume, max(0, b_xfer - spent))
        if rc == B.KV_ENOSPC:                     # copied-out blocks are not reusable within the call
            resume = []
            rc, n_eager = tab.kv_table_rotate_eager(pre, [], max(0, b_xfer - len(pre)))
        assert rc == 0, B.kv_strerror(rc)
        sched_ms = (time.perf_counter() - h0) * 1e3      # LVF, the fit, the table's work and the enqueue
        assert eng.kv_wait() == 0
        prep_ms = (time.perf_counter() - x0) * 1e3       # scheduling + transfer, from the start of the execution
        st = eng.kv_last_stats()
        rc, _, pm = eng.kv_reader_wait()
        assert rc == 0
        exec_ms = float(sum(pm))
        moved = (st["bytes_out"] + st["bytes_in"]) // blk
        moved_blocks += moved
        t_sched.append(sched_ms)
        t_exec.append(exec_ms)
        if moved:
            n_rot += 1
            t_xfer.append(st["ms_e2e"])                  # the engine's clock: transfer call entry to kv_wait return
            t_prep.append(prep_ms)
            n_stall += prep_ms > exec_ms
        if fixed_budget is None:
            b_xfer = max(8, int(0.8 * 48e9 * float(np.mean(t_exec[-32:])) * 1e-3 / blk))
        now += max(exec_ms, prep_ms) * 1e-3
        it += 1
        # ---- bookkeeping of what was decided -----------------------------------------------------------
        started = []
        for r in admit:
            rc, new = tab.kv_table_append(r, length[r])
            if rc != 0:
                continue
            state[r], t_ref[r] = B.KV_REQ_RUNNING, now
            started.append(r)
        for r in pre:
            state[r], t_ref[r] = B.KV_REQ_ROTARY, t_ref.get(("last", r), now)
        for r in resume:
            state[r], t_ref[r] = B.KV_REQ_RUNNING, now
        # ---- every request of the batch (and every admitted prompt) yields one token ----------------
        for r in batch + started:
            if state.get(r) != B.KV_REQ_RUNNING:
                continue
            if r not in first_done:
                first_done.add(r)
                ttft.append(now - arrive_time[r])
            else:
                tbt.append(now - t_ref[("last", r)])
            t_ref[("last", r)] = now
            length[r] += 1
            if length[r] >= target[r]:
                assert eng.kv_wait() == 0
                assert tab.kv_table_finish(r) == 0
                for d in (state, length, target):
                    d.pop(r, None)
                t_ref.pop(r, None); t_ref.pop(("last", r), None)
                first_done.discard(r)
                free_ids.append(r)
                continue
            rc, new = tab.kv_table_append(r, 1)
            if rc != 0:
                length[r] -= 1                    # cache full: the token waits for the next iteration
    # every synced block must still equal its DRAM copy
    assert eng.kv_wait() == 0
    pool = eng.host_pool_array().view(np.uint16).reshape((shape.n_host_slots,) + shape.block_dims())
    checked = 0
    for r in [r for r in state if state[r] == B.KV_REQ_RUNNING][:24]:
        b = tab.kv_table_blocks(r)
        if b is None:
            continue
        sel = [i for i, s_ in enumerate(b["states"]) if s_ == B.KV_BLOCK_SYNCED][:8]
        if not sel:
            continue
        hb = cache.view(torch.int16)[:, :, torch.tensor([b["ids"][i] for i in sel], device="cuda")].cpu().numpy()
        assert np.array_equal(hb.view(np.uint16).transpose(2, 0, 1, 3, 4, 5), pool[[b["slots"][i] for i in sel]])
        checked += len(sel)
    c = tab.kv_table_get_counts()
    q = lambda a, p_: float(np.percentile(a, p_)) if len(a) else float("nan")
    print(f"\nsynthetic serving, {rps:g} requests/s for {seconds:g} s of virtual time, execution = {exec_passes} x 16 GiB read, "
          f"B_xfer = {b_xfer} blocks "
          f"({b_xfer * blk / 2**20:.0f} MiB) per iteration{'' if fixed_budget is not None else ' (0.8 x link rate x execution time)'}, "
          f"HBM cache {shape.n_hbm_blocks} blocks, {len(state)} requests still in flight\n")
    print("| iterations | with a rotation | stalled (scheduling + transfer outlasted execution) | schedule ms avg | "
          "transfer ms avg (engine clock) | schedule + transfer ms avg, p99 | execution ms avg | blocks moved | eager copies | "
          "copied at preemption | dropped without copy | swapped in |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|")
    print(f"| {it} | {n_rot} | {n_stall} ({100.0 * n_stall / max(it, 1):.2f} % of iterations) | {np.mean(t_sched):.2f} | "
          f"{np.mean(t_xfer) if t_xfer else 0:.2f} | {np.mean(t_prep) if t_prep else 0:.2f}, {q(t_prep, 99):.2f} | "
          f"{np.mean(t_exec):.2f} | {moved_blocks} | {c['copied_eager']} | "
          f"{c['copied_preempt']} | {c['dropped_synced']} | {c['swapped_in']} |")
    print(f"\nTTFT p50 / p99: {q(ttft, 50):.3f} / {q(ttft, 99):.3f} s over {len(ttft)} requests; "
          f"TBT p50 / p99: {q(tbt, 50) * 1e3:.1f} / {q(tbt, 99) * 1e3:.1f} ms over {len(tbt)} tokens; "
          f"{checked} synced blocks re-checked against their DRAM copies")
    tab.kv_table_destroy()
    eng.kv_destroy()
    return dict(iterations=it, stalled=n_stall, counts=c, checked=checked, in_flight=len(state))


if __name__ == "__main__":
    what = sys.argv[1] if len(sys.argv) > 1 else "configs"
    if what == "serve" and len(sys.argv) > 2:
        serve(rps=float(sys.argv[2]), seconds=float(sys.argv[3]) if len(sys.argv) > 3 else 20.0,
              exec_passes=int(sys.argv[4]) if len(sys.argv) > 4 else 1)
        sys.exit(0)
    {"ladder": ladder, "configs": configs, "interference": interference, "reader": reader,
     "eager": eager, "layouts": layouts,
     "linksweep": linksweep, "serve": serve,
     "sizes": sizes, "ratio": ratio, "chunks": chunks, "layers": layers, "poolkinds": poolkinds, "splitcalls": splitcalls, "packalone": packalone,
     "packshapes": packshapes}[what]()
