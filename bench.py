"""Benchmark of the duplex KV rotation on one MI355X.

One "step" is one full rotation of the workload through the hot path:
admission, descriptor upload, the transfer kernels / copies in both
directions, and completion (kv_rotate + kv_wait).  Steps alternate between the
rotation and its inverse so the cache and pool return to their initial state.

Prints ONE JSON line on stdout; everything else goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PCIE5_X16_PER_DIR_GBPS = 64.0   # 32 GT/s x 16 lanes / 8, raw, per direction
HBM_PEAK_GBPS = 8000.0



def measured_traffic(workload, path, kernel):
    """Bytes through L2<->fabric per launch of `kernel`, from rocprofv3 --pmc
    FETCH_SIZE and WRITE_SIZE runs of this script scaled by the plain copy of
    --calibrate-copy.  The summaries under profiles/ carry one line per figure,
        bench-traffic workload=<w> path=<p> kernel=<k> bytes_per_launch=<n>
    and this looks the line up; (None, None) when no summary covers the run.
    The counters see HBM and host-memory accesses alike: each moved byte is read
    once and written once, so the algorithmic figure of the move kernel is
    2 x (bytes_out + bytes_in)."""
    pdir = os.path.join(ROOT, "profiles")
    want = {"workload": workload, "path": path, "kernel": kernel}
    for name in sorted(os.listdir(pdir)) if os.path.isdir(pdir) else []:
        if not name.endswith((".txt", ".md")):
            continue
        for line in open(os.path.join(pdir, name)):
            if not line.startswith("bench-traffic "):
                continue
            kv = dict(f.split("=", 1) for f in line.split()[1:] if "=" in f)
            if all(kv.get(k) == v for k, v in want.items()) and kv.get("bytes_per_launch", "").isdigit():
                return int(kv["bytes_per_launch"]), "profiles/" + name
    return None, None


def host_topology():
    """NUMA nodes with their CPU lists, and the CPUs this process may run on."""
    nodes = {}
    base = "/sys/devices/system/node"
    try:
        for d in sorted(os.listdir(base)):
            if d.startswith("node") and d[4:].isdigit():
                nodes[d] = open(os.path.join(base, d, "cpulist")).read().strip()
    except OSError:
        pass
    try:
        allowed = sorted(os.sched_getaffinity(0))
    except AttributeError:
        allowed = list(range(os.cpu_count() or 1))
    return nodes, allowed


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(shape, rot, layout, budget_s=12.0):
    """The oracle, as it stands, on host arrays shaped like the workload."""
    import numpy as np
    from oracle import kv_oracle as O
    s = O.shape_of(shape, layout)
    blk = O.block_bytes(s)
    # untouched pages of these arrays are never made resident
    hbm = np.empty(O.cache_bytes(s), dtype=np.uint8)
    pool = np.empty(O.pool_bytes(s), dtype=np.uint8)
    rng = np.random.default_rng(1)
    seg = O.seg_bytes(s)
    fill = rng.integers(0, 256, seg, dtype=np.uint8)
    for l in range(shape.n_layers):
        for kv in range(2):
            for b in list(rot.out_ids) + list(rot.in_ids):
                o = O.hbm_offset(s, l, kv, int(b)); hbm[o:o + seg] = fill
            for sl in list(rot.out_slots) + list(rot.in_slots):
                o = O.pool_offset(s, l, kv, int(sl)); pool[o:o + seg] = fill
    inv = rot.inverse()
    moved = (len(rot.out_ids) + len(rot.in_ids)) * blk
    out = {}
    nodes, allowed = host_topology()
    for label, threads in (("single", 0), ("all", len(allowed))):
        for r in (rot, inv):  # warm
            O.rotate(s, hbm, pool, r.out_ids, r.out_slots, r.in_ids, r.in_slots, threads=threads)
        n, t0 = 0, time.perf_counter()
        while time.perf_counter() - t0 < budget_s / 2:
            for r in (rot, inv):
                rc = O.rotate(s, hbm, pool, r.out_ids, r.out_slots, r.in_ids, r.in_slots, threads=threads)
                assert rc == 0
            n += 2
        dt = time.perf_counter() - t0
        out[label] = (moved * n / dt / 1e9, n, max(threads, 1))
    return {"value": round(out["all"][0], 2), "unit": "GB/s", "cores": out["all"][2], "kind": "oracle",
            "sample": f"{out['all'][1]} rotations of the same id lists on pageable host arrays "
                      f"({moved >> 20} MiB moved each), threads split the block lists",
            "single_thread_value": round(out["single"][0], 2),
            "numa_nodes": nodes, "cpus_allowed": ",".join(map(str, allowed))}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="llama3_8b")
    ap.add_argument("--path", default="auto", choices=["auto", "sdma_staged", "zerocopy", "naive", "fused"])
    ap.add_argument("--layout", default="block_first", choices=["block_first", "layer_first"])
    ap.add_argument("--contiguous-slots", action="store_true")
    ap.add_argument("--max-copy-wgs", type=int, default=0)
    ap.add_argument("--chunk-layers", type=int, default=0)
    ap.add_argument("--staging-mib", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy kernel, the known-size reference for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (KV rotation never crosses GPUs); use --gpus 1")

    import numpy as np
    import torch
    from paper_2601_20309_amd import binding as B
    from paper_2601_20309_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    shape = W.SHAPES[args.workload]
    layout = {"block_first": B.KV_HOST_BLOCK_FIRST, "layer_first": B.KV_HOST_LAYER_FIRST}[args.layout]
    path = {v: k for k, v in B.PATH_NAMES.items()}[args.path]
    rot = W.config_rotation(args.workload, contiguous_slots=args.contiguous_slots)
    inv = rot.inverse()
    cfg = B.make_config(shape, layout, path, chunk_layers=args.chunk_layers,
                        max_copy_wgs=args.max_copy_wgs, staging_bytes=args.staging_mib << 20)
    blk = B.kv_block_bytes(cfg)
    log(f"workload {args.workload}: cache {B.kv_cache_bytes(cfg) / 2**30:.1f} GiB, pool "
        f"{B.kv_pool_bytes(cfg) / 2**30:.1f} GiB, {len(rot.out_ids)} blocks out + {len(rot.in_ids)} in "
        f"({blk >> 10} KiB each)")

    # the denominator first, while no other stream exists in the process (streams
    # share a small number of hardware queues; two that share one serialise)
    # per direction: the best median over 64 MiB, 256 MiB and 1 GiB copies
    link, link_by_size = {}, {}
    for mib in (64, 256, 1024):
        r = B.kv_probe_link(mib << 20, 5)
        link_by_size[f"{mib}MiB"] = {k: round(v, 2) for k, v in r.items()}
        log(f"hipMemcpyAsync pinned {mib} MiB: " + ", ".join(f"{k} {v:.2f} GB/s" for k, v in r.items()))
        for k, v in r.items():
            link[k] = max(link.get(k, 0.0), v)

    t = time.time()
    cache = W.cache_image(shape, W.value_seed(args.workload), device="cuda")
    torch.cuda.synchronize()
    eng = B.Engine(cfg, cache.data_ptr())
    pool = eng.host_pool_array()
    # stage the incoming request's blocks in its slots (through the documented pool layout)
    staged = W.staged_blocks(shape, len(rot.in_slots), W.value_seed(args.workload) + 50, device="cuda")
    staged_np = staged.view(torch.int16).cpu().numpy().view(np.uint16)
    if layout == B.KV_HOST_BLOCK_FIRST:
        pv = pool.view(np.uint16).reshape((shape.n_host_slots,) + shape.block_dims())
        pv[rot.in_slots] = staged_np
    else:
        pv = pool.view(np.uint16).reshape(shape.n_layers, 2, shape.n_host_slots, shape.block_size,
                                          shape.n_kv_heads, shape.head_dim)
        pv[:, :, rot.in_slots] = staged_np.transpose(1, 2, 0, 3, 4, 5)
    log(f"setup {time.time() - t:.1f} s")

    calls = (eng.prepare(rot.out_ids, rot.out_slots, rot.in_ids, rot.in_slots),
             eng.prepare(inv.out_ids, inv.out_slots, inv.in_ids, inv.in_slots))

    def step(i):
        rc = calls[i & 1]()
        assert rc == 0, B.kv_strerror(rc)
        rc = eng.kv_wait()
        assert rc == 0, B.kv_strerror(rc)

    # expected first-step result from the oracle, on the named blocks only
    if not args.no_check:
        cv = cache.view(torch.int16)
        before_out = cv[:, :, torch.from_numpy(rot.out_ids).long().cuda()].cpu()   # [L,2,n,P,H,D]
    for i in range(args.warmup + (args.warmup % 2)):   # even count: state returns
        step(i)
        if i == 0 and not args.no_check:
            # swapped-in blocks must now hold the staged bytes; slots the swapped-out ones
            got_in = cv[:, :, torch.from_numpy(rot.in_ids).long().cuda()].cpu()
            assert torch.equal(got_in, staged.view(torch.int16).cpu().permute(1, 2, 0, 3, 4, 5)), "swap-in mismatch"
            if layout == B.KV_HOST_BLOCK_FIRST:
                got_out = torch.from_numpy(pv[rot.out_slots].view(np.int16)).permute(1, 2, 0, 3, 4, 5)
            else:
                got_out = torch.from_numpy(pv[:, :, rot.out_slots].view(np.int16))
            assert torch.equal(got_out, before_out), "swap-out mismatch"
            log("first step verified against the staged and original blocks")

    if args.calibrate_copy:
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_()
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    steps = args.steps + (args.steps % 2)
    ms_out = ms_in = 0.0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    per_step = []
    for i in range(steps):
        ts = time.perf_counter()
        step(i)
        per_step.append(time.perf_counter() - ts)
        st = eng.kv_last_stats()
        ms_out += st["ms_out"]; ms_in += st["ms_in"]
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    st = eng.kv_last_stats()
    bytes_out, bytes_in = len(rot.out_ids) * blk, len(rot.in_ids) * blk
    ms_step = dt / steps * 1e3
    gbps_out = bytes_out / (ms_step * 1e6)
    gbps_in = bytes_in / (ms_step * 1e6)
    kern_ms = max(ms_out, ms_in) / steps

    if not args.no_check:
        # full-cache property: after an even number of steps every block holds its
        # original bytes, except the swap-in targets, which keep the staged blocks
        again = W.cache_image(shape, W.value_seed(args.workload), device="cuda")
        again[:, :, torch.from_numpy(rot.in_ids).long().cuda()] = staged.permute(1, 2, 0, 3, 4, 5)
        assert torch.equal(again.view(torch.int16), cache.view(torch.int16)), "cache image wrong after the loop"
        del again
        log("whole cache verified after the timed loop")

    path_name = B.PATH_NAMES[st["path_used"]]
    # the kernel of the step: the move kernel, or, on the DMA-staged path, the pack / unpack kernel
    # (its bench-traffic line is per launch of that kernel, one chunk)
    traffic, traffic_src = measured_traffic(args.workload, path_name,
                                            "kv_stage_kernel" if path_name == "sdma_staged" else "kv_move_kernel")
    res = {
        "metric": "duplex KV rotation GB/s (out+in) and % of measured host-link peak",
        "value": round(gbps_out + gbps_in, 2), "unit": "GB/s", "n_gpus": 1, "steps": steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4),
        "ms_per_step_median": round(float(np.median(per_step)) * 1e3, 4),
        "ms_per_step_min": round(min(per_step) * 1e3, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {shape.n_layers} layers x {shape.n_kv_heads} KV heads x "
                               f"{shape.head_dim} dims, block {shape.block_size}, bf16 N(0,1); "
                               f"{shape.n_hbm_blocks} HBM blocks, {shape.n_host_slots} host slots; "
                               f"{len(rot.out_ids)} scattered blocks out while {len(rot.in_ids)} in",
                   "path": B.PATH_NAMES[st["path_used"]], "host_layout": args.layout,
                   "contiguous_slots": bool(args.contiguous_slots),
                   "bytes_out": bytes_out, "bytes_in": bytes_in, "launches_per_step": st["n_launches"]},
        "gbps_out": round(gbps_out, 2), "gbps_in": round(gbps_in, 2),
        "link_peak_memcpy": {k: round(v, 2) for k, v in link.items()},
        "link_peak_memcpy_by_size": link_by_size,
        "pct_of_peak_out": round(100 * gbps_out / link["d2h"], 1),
        "pct_of_peak_in": round(100 * gbps_in / link["h2d"], 1),
        "roofline": {
            "bound": "host_link", "kernel": "kv_move_kernel (both directions in one launch)"
            if st["path_used"] == B.KV_PATH_FUSED else B.PATH_NAMES[st["path_used"]],
            "achieved": round((bytes_out + bytes_in) / (kern_ms * 1e6), 2),
            "peak": 2 * PCIE5_X16_PER_DIR_GBPS, "unit": "GB/s",
            "frac": round((bytes_out + bytes_in) / (kern_ms * 1e6) / (2 * PCIE5_X16_PER_DIR_GBPS), 4),
            "frac_of_measured_memcpy_peak": round((bytes_out + bytes_in) / (kern_ms * 1e6) /
                                                  (link["d2h"] + link["h2d"]), 4),
            "kernel_ms": round(kern_ms, 4),
            "traffic": traffic, "profile": traffic_src,
            # per launch: the move kernel reads and writes both directions' bytes once; a pack or
            # unpack launch reads and writes one direction's
            "traffic_algorithmic": 2 * bytes_out if path_name == "sdma_staged" else 2 * (bytes_out + bytes_in),
            "hbm_frac": round((bytes_out + bytes_in) / (kern_ms * 1e6) / HBM_PEAK_GBPS, 5),
        },
    }
    # the hot path's HBM-bound kernel (the decode reader that runs beside rotations), measured
    # live on its own stream with HIP events: every block of the cache, 6 passes
    all_ids = np.arange(shape.n_hbm_blocks, dtype=np.int32)
    assert eng.kv_reader_start(all_ids, 6) == 0
    rc, _, pass_ms = eng.kv_reader_wait()
    assert rc == 0
    rd_ms = float(np.median(pass_ms[1:]))
    rd_bytes = shape.n_hbm_blocks * blk
    rd_traffic, rd_src = measured_traffic(args.workload, "reader", "kv_reader_kernel")
    res["roofline_hbm_kernel"] = {
        "bound": "hbm", "kernel": "kv_reader_kernel (synthetic decode reader, whole cache per launch)",
        "achieved": round(rd_bytes / (rd_ms * 1e6), 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(rd_bytes / (rd_ms * 1e6) / HBM_PEAK_GBPS, 4), "kernel_ms": round(rd_ms, 4),
        "traffic": rd_traffic, "profile": rd_src, "traffic_algorithmic": rd_bytes,
    }
    eng.kv_destroy()
    del cache
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(shape, rot, layout)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
