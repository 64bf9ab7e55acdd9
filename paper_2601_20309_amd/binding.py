"""Thin ctypes binding of libduplexkv.so: same names as include/duplexkv.h,
argument marshalling only.  Every byte is moved by the library's HIP code;
there is no fallback: if the library is missing, importing this fails loudly."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
# PyTorch ships its own HIP runtime.  It must be in the process before this
# library is loaded so that both resolve to the same libamdhip64 (two runtimes
# in one process do not see the device); torch also owns the cache allocation.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libduplexkv.so")

KV_OK, KV_EINVAL, KV_ERANGE, KV_EDUP, KV_EOVERLAP, KV_ENOMEM, KV_EHIP, KV_EUNSUP, KV_ENOSPC, KV_EBUSY, KV_E2BIG = \
    0, -1, -2, -3, -4, -5, -6, -7, -8, -9, -10
KV_STATIC_MAX_BLOCKS = 8192
KV_BLOCK_DIRTY, KV_BLOCK_FULL, KV_BLOCK_SYNCED, KV_BLOCK_HOST = 1, 2, 3, 4
KV_HOST_BLOCK_FIRST, KV_HOST_LAYER_FIRST = 0, 1
KV_HBM_LAYER_FIRST, KV_HBM_BLOCK_FIRST = 0, 1
KV_PATH_AUTO, KV_PATH_SDMA_STAGED, KV_PATH_ZEROCOPY, KV_PATH_NAIVE, KV_PATH_FUSED, KV_PATH_DMA_BLOCKS = \
    0, 1, 2, 3, 4, 5
PATH_NAMES = {0: "auto", 1: "sdma_staged", 2: "zerocopy", 3: "naive", 4: "fused", 5: "dma_blocks"}

EXPORTS = ["kv_seg_bytes", "kv_block_bytes", "kv_cache_bytes", "kv_pool_bytes", "kv_validate",
           "kv_create", "kv_destroy", "kv_swap_out", "kv_swap_in", "kv_rotate", "kv_rotate_static", "kv_wait", "kv_query", "kv_stream_wait_layer", "kv_wait_layer",
           "kv_host_pool", "kv_last_stats", "kv_probe_link", "kv_reader_start", "kv_reader_wait",
           "kv_table_create", "kv_table_destroy", "kv_table_append", "kv_table_eager", "kv_table_rotate", "kv_table_rotate_eager",
           "kv_table_finish", "kv_table_blocks", "kv_table_get_counts", "kv_sched_vlt", "kv_sched_lvf",
           "kv_strerror"]
KV_REQ_RUNNING, KV_REQ_WAITING, KV_REQ_ROTARY = 0, 1, 2


class kv_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "n_kv_heads", "head_dim", "block_size", "elem_bytes", "n_hbm_blocks",
        "n_host_slots", "host_layout", "path", "chunk_layers", "max_copy_wgs", "vecs_per_lane", "wg_lanes", "hbm_layout")] + \
        [("staging_bytes", C.c_uint64)]


class kv_stats(C.Structure):
    _fields_ = [("bytes_out", C.c_uint64), ("bytes_in", C.c_uint64), ("ms_out", C.c_double),
                ("ms_in", C.c_double), ("ms_e2e", C.c_double), ("path_used", C.c_int32),
                ("n_launches", C.c_int32)]


class kv_table_counts(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("free_hbm_blocks", "free_host_slots", "copied_eager",
                                         "copied_preempt", "dropped_synced", "swapped_in")]


class kv_sched_params(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("alpha", "beta_b", "beta_f", "slo_tbt", "slo_ttft")]


class kv_sched_req(C.Structure):
    _fields_ = [("id", C.c_int32), ("state", C.c_int32), ("blocks", C.c_int32), ("pad", C.c_int32),
                ("t_ref", C.c_double)]


class KVError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {kv_strerror(code)} ({code})")
        self.code = code


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is not built; run `python -m paper_2601_20309_amd.build` "
            "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    p32, pcfg = C.POINTER(C.c_int32), C.POINTER(kv_config)
    for n in ("kv_seg_bytes", "kv_block_bytes", "kv_cache_bytes", "kv_pool_bytes"):
        getattr(L, n).restype = C.c_uint64
        getattr(L, n).argtypes = [pcfg]
    L.kv_validate.restype = C.c_int
    L.kv_validate.argtypes = [pcfg, p32, p32, C.c_int32, p32, p32, C.c_int32]
    L.kv_create.restype = C.c_int
    L.kv_create.argtypes = [C.POINTER(C.c_void_p), pcfg, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.kv_destroy.restype = C.c_int
    L.kv_destroy.argtypes = [C.c_void_p]
    L.kv_swap_out.restype = C.c_int
    L.kv_swap_out.argtypes = [C.c_void_p, p32, p32, C.c_int32]
    L.kv_swap_in.restype = C.c_int
    L.kv_swap_in.argtypes = [C.c_void_p, p32, p32, C.c_int32]
    L.kv_rotate.restype = C.c_int
    L.kv_rotate.argtypes = [C.c_void_p, p32, p32, C.c_int32, p32, p32, C.c_int32]
    L.kv_rotate_static.restype = C.c_int
    L.kv_rotate_static.argtypes = [pcfg, C.c_void_p, C.c_void_p, C.c_void_p, p32, p32, C.c_int32, p32, p32, C.c_int32]
    L.kv_wait.restype = C.c_int
    L.kv_wait.argtypes = [C.c_void_p]
    L.kv_query.restype = C.c_int
    L.kv_query.argtypes = [C.c_void_p]
    L.kv_stream_wait_layer.restype = C.c_int
    L.kv_stream_wait_layer.argtypes = [C.c_void_p, C.c_void_p, C.c_int32]
    L.kv_wait_layer.restype = C.c_int
    L.kv_wait_layer.argtypes = [C.c_void_p, C.c_int32]
    L.kv_host_pool.restype = C.c_int
    L.kv_host_pool.argtypes = [C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_uint64)]
    L.kv_last_stats.restype = C.c_int
    L.kv_last_stats.argtypes = [C.c_void_p, C.POINTER(kv_stats)]
    L.kv_probe_link.restype = C.c_int
    L.kv_probe_link.argtypes = [C.c_uint64, C.c_int32] + [C.POINTER(C.c_double)] * 4
    L.kv_reader_start.restype = C.c_int
    L.kv_reader_start.argtypes = [C.c_void_p, p32, C.c_int32, C.c_int32, C.c_int32]
    L.kv_reader_wait.restype = C.c_int
    L.kv_reader_wait.argtypes = [C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_double)]
    L.kv_table_create.restype = C.c_int
    L.kv_table_create.argtypes = [C.POINTER(C.c_void_p), C.c_void_p, C.c_int32]
    L.kv_table_destroy.restype = C.c_int
    L.kv_table_destroy.argtypes = [C.c_void_p]
    L.kv_table_append.restype = C.c_int
    L.kv_table_append.argtypes = [C.c_void_p, C.c_int32, C.c_int32, p32, C.c_int32, p32]
    L.kv_table_eager.restype = C.c_int
    L.kv_table_eager.argtypes = [C.c_void_p, C.c_int32, p32]
    L.kv_table_rotate.restype = C.c_int
    L.kv_table_rotate.argtypes = [C.c_void_p, p32, C.c_int32, p32, C.c_int32]
    L.kv_table_rotate_eager.restype = C.c_int
    L.kv_table_rotate_eager.argtypes = [C.c_void_p, p32, C.c_int32, p32, C.c_int32, C.c_int32, p32]
    L.kv_table_finish.restype = C.c_int
    L.kv_table_finish.argtypes = [C.c_void_p, C.c_int32]
    L.kv_table_blocks.restype = C.c_int
    L.kv_table_blocks.argtypes = [C.c_void_p, C.c_int32, p32, p32, p32, C.c_int32, p32, p32]
    L.kv_table_get_counts.restype = C.c_int
    L.kv_table_get_counts.argtypes = [C.c_void_p, C.POINTER(kv_table_counts)]
    L.kv_sched_vlt.restype = C.c_double
    L.kv_sched_vlt.argtypes = [C.POINTER(kv_sched_params), C.POINTER(kv_sched_req), C.c_double]
    L.kv_sched_lvf.restype = C.c_int
    L.kv_sched_lvf.argtypes = [C.POINTER(kv_sched_params), C.POINTER(kv_sched_req), C.c_int32, C.c_double,
                               C.c_int32, C.c_int32, p32, p32, p32, p32, p32]
    L.kv_strerror.restype = C.c_char_p
    L.kv_strerror.argtypes = [C.c_int]
    return L


lib = _load()


def make_config(shape, host_layout=KV_HOST_BLOCK_FIRST, path=KV_PATH_AUTO, chunk_layers=0,
                max_copy_wgs=0, staging_bytes=0, vecs_per_lane=0, wg_lanes=0, hbm_layout=KV_HBM_LAYER_FIRST) -> kv_config:
    """kv_config from any object carrying the KV shape attributes."""
    return kv_config(shape.n_layers, shape.n_kv_heads, shape.head_dim, shape.block_size,
                     shape.elem_bytes, shape.n_hbm_blocks, shape.n_host_slots, host_layout, path,
                     chunk_layers, max_copy_wgs, vecs_per_lane, wg_lanes, hbm_layout, staging_bytes)


def _ids(a):
    if a is None:
        return None, 0, None
    arr = np.ascontiguousarray(a, dtype=np.int32)
    if arr.size == 0:
        return None, 0, arr
    return arr.ctypes.data_as(C.POINTER(C.c_int32)), int(arr.size), arr


def kv_strerror(code: int) -> str:
    return lib.kv_strerror(code).decode()


def kv_seg_bytes(cfg): return int(lib.kv_seg_bytes(C.byref(cfg)))
def kv_block_bytes(cfg): return int(lib.kv_block_bytes(C.byref(cfg)))
def kv_cache_bytes(cfg): return int(lib.kv_cache_bytes(C.byref(cfg)))
def kv_pool_bytes(cfg): return int(lib.kv_pool_bytes(C.byref(cfg)))


def kv_validate(cfg, out_block_ids, out_host_slots, in_block_ids, in_host_slots,
                n_out: Optional[int] = None, n_in: Optional[int] = None) -> int:
    po, no, k1 = _ids(out_block_ids); ps, no2, k2 = _ids(out_host_slots)
    pi, ni, k3 = _ids(in_block_ids); pis, ni2, k4 = _ids(in_host_slots)
    assert no == no2 and ni == ni2
    return lib.kv_validate(C.byref(cfg), po, ps, no if n_out is None else n_out,
                           pi, pis, ni if n_in is None else n_in)


def kv_rotate_static(cfg, hbm_cache_ptr: int, host_pool_ptr: int, stream: int,
                     out_block_ids, out_host_slots, in_block_ids, in_host_slots) -> int:
    po, no, k1 = _ids(out_block_ids); ps, no2, k2 = _ids(out_host_slots)
    pi, ni, k3 = _ids(in_block_ids); pis, ni2, k4 = _ids(in_host_slots)
    assert no == no2 and ni == ni2
    return lib.kv_rotate_static(C.byref(cfg), C.c_void_p(hbm_cache_ptr or None), C.c_void_p(host_pool_ptr or None),
                                C.c_void_p(stream or None), po, ps, no, pi, pis, ni)


def kv_probe_link(nbytes: int, reps: int = 5) -> dict:
    v = [C.c_double() for _ in range(4)]
    rc = lib.kv_probe_link(nbytes, reps, *[C.byref(x) for x in v])
    if rc != KV_OK:
        raise KVError(rc, "kv_probe_link")
    return dict(d2h=v[0].value, h2d=v[1].value, d2h_duplex=v[2].value, h2d_duplex=v[3].value)


def kv_sched_vlt(params, req, t_now: float) -> float:
    """params = (alpha, beta_b, beta_f, slo_tbt, slo_ttft); req = (id, state, blocks, t_ref)."""
    p = kv_sched_params(*params)
    r = kv_sched_req(req[0], req[1], req[2], 0, req[3])
    return lib.kv_sched_vlt(C.byref(p), C.byref(r), t_now)


def kv_sched_lvf(params, reqs, t_now: float, b_xfer: int, b_hbm: int):
    """(code, preempted ids, prioritised ids, fcfs flag)."""
    p = kv_sched_params(*params)
    n = len(reqs)
    arr = (kv_sched_req * max(n, 1))(*[kv_sched_req(r[0], r[1], r[2], 0, r[3]) for r in reqs])
    pre, pri = (C.c_int32 * max(n, 1))(), (C.c_int32 * max(n, 1))()
    npre, npri, fcfs = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    rc = lib.kv_sched_lvf(C.byref(p), arr, n, t_now, b_xfer, b_hbm, pre, C.byref(npre), pri, C.byref(npri),
                          C.byref(fcfs))
    return rc, list(pre[:npre.value]), list(pri[:npri.value]), bool(fcfs.value)


class Engine:
    """Owns one kv_engine handle.  Methods carry the C names and return the C
    result code (raise_on_error=False) or raise KVError."""

    def __init__(self, cfg: kv_config, hbm_cache_ptr: int, host_pool_ptr: int = 0,
                 stream_out: int = 0, stream_in: int = 0):
        self.cfg = cfg
        self._h = C.c_void_p()
        rc = lib.kv_create(C.byref(self._h), C.byref(cfg), C.c_void_p(hbm_cache_ptr),
                           C.c_void_p(host_pool_ptr or None), C.c_void_p(stream_out or None),
                           C.c_void_p(stream_in or None))
        if rc != KV_OK:
            self._h = C.c_void_p()
            raise KVError(rc, "kv_create")

    def kv_swap_out(self, block_ids, host_slots) -> int:
        pi, n, k1 = _ids(block_ids); ps, n2, k2 = _ids(host_slots)
        assert n == n2
        return lib.kv_swap_out(self._h, pi, ps, n)

    def kv_swap_in(self, host_slots, block_ids) -> int:
        ps, n, k1 = _ids(host_slots); pi, n2, k2 = _ids(block_ids)
        assert n == n2
        return lib.kv_swap_in(self._h, ps, pi, n)

    def kv_rotate(self, out_block_ids, out_host_slots, in_block_ids, in_host_slots) -> int:
        po, no, k1 = _ids(out_block_ids); ps, no2, k2 = _ids(out_host_slots)
        pi, ni, k3 = _ids(in_block_ids); pis, ni2, k4 = _ids(in_host_slots)
        assert no == no2 and ni == ni2
        return lib.kv_rotate(self._h, po, ps, no, pi, pis, ni)

    def prepare(self, out_block_ids, out_host_slots, in_block_ids, in_host_slots):
        """Marshal one rotation's id lists once; returns a zero-argument callable
        that performs the kv_rotate call (for loops that repeat a rotation)."""
        po, no, k1 = _ids(out_block_ids); ps, no2, k2 = _ids(out_host_slots)
        pi, ni, k3 = _ids(in_block_ids); pis, ni2, k4 = _ids(in_host_slots)
        assert no == no2 and ni == ni2
        h, f = self._h, lib.kv_rotate

        def call(_keep=(k1, k2, k3, k4)):
            return f(h, po, ps, no, pi, pis, ni)
        return call

    def kv_wait(self) -> int:
        return lib.kv_wait(self._h)

    def kv_query(self) -> int:
        return lib.kv_query(self._h)

    def kv_stream_wait_layer(self, stream: int, layer: int) -> int:
        return lib.kv_stream_wait_layer(self._h, C.c_void_p(stream or None), layer)

    def kv_wait_layer(self, layer: int) -> int:
        return lib.kv_wait_layer(self._h, layer)

    def kv_host_pool(self):
        ptr, n = C.c_void_p(), C.c_uint64()
        rc = lib.kv_host_pool(self._h, C.byref(ptr), C.byref(n))
        if rc != KV_OK:
            raise KVError(rc, "kv_host_pool")
        return ptr.value, n.value

    def host_pool_array(self) -> np.ndarray:
        """The pool as a uint8 NumPy array over the pinned memory (no copy)."""
        ptr, n = self.kv_host_pool()
        buf = (C.c_uint8 * n).from_address(ptr)
        return np.frombuffer(buf, dtype=np.uint8)

    def kv_last_stats(self) -> dict:
        st = kv_stats()
        rc = lib.kv_last_stats(self._h, C.byref(st))
        if rc != KV_OK:
            raise KVError(rc, "kv_last_stats")
        return {f: getattr(st, f) for f, _ in kv_stats._fields_}

    def kv_reader_start(self, block_ids, passes: int = 1, max_wgs: int = 0) -> int:
        pi, n, k1 = _ids(block_ids)
        self._reader_passes = passes
        return lib.kv_reader_start(self._h, pi, n, passes, max_wgs)

    def kv_reader_wait(self):
        """(code, checksum over all passes, [ms of each pass])."""
        n = getattr(self, "_reader_passes", 0)
        ms = (C.c_double * max(n, 1))()
        cs = C.c_uint64(0)
        rc = lib.kv_reader_wait(self._h, C.byref(cs), ms)
        return rc, int(cs.value), [ms[i] for i in range(n)]

    def kv_destroy(self) -> int:
        if self._h:
            rc = lib.kv_destroy(self._h)
            if rc != KV_EBUSY:      # refused while a block table is attached: the handle stays valid
                self._h = C.c_void_p()
            return rc
        return KV_OK

    def __del__(self):
        try:
            self.kv_destroy()
        except Exception:
            pass


class Table:
    """Owns one kv_table handle on top of an Engine (same names as the C ABI)."""

    def __init__(self, engine: Engine, max_requests: int):
        self.engine = engine
        self._cap = int(engine.cfg.n_hbm_blocks)
        self._h = C.c_void_p()
        rc = lib.kv_table_create(C.byref(self._h), engine._h, max_requests)
        if rc != KV_OK:
            self._h = C.c_void_p()
            raise KVError(rc, "kv_table_create")

    def kv_table_append(self, req: int, n_tokens: int):
        """(code, [newly allocated HBM block ids])."""
        ids = (C.c_int32 * self._cap)()
        n = C.c_int32(0)
        rc = lib.kv_table_append(self._h, req, n_tokens, ids, self._cap, C.byref(n))
        return rc, [ids[i] for i in range(n.value)] if rc == KV_OK else []

    def kv_table_eager(self, budget: int):
        n = C.c_int32(0)
        rc = lib.kv_table_eager(self._h, budget, C.byref(n))
        return rc, n.value

    def kv_table_rotate(self, preempt, resume) -> int:
        pp, np_, k1 = _ids(preempt)
        pr, nr, k2 = _ids(resume)
        return lib.kv_table_rotate(self._h, pp, np_, pr, nr)

    def kv_table_rotate_eager(self, preempt, resume, eager_budget: int):
        pp, np_, k1 = _ids(preempt)
        pr, nr, k2 = _ids(resume)
        n = C.c_int32(0)
        rc = lib.kv_table_rotate_eager(self._h, pp, np_, pr, nr, eager_budget, C.byref(n))
        return rc, n.value

    def kv_table_finish(self, req: int) -> int:
        return lib.kv_table_finish(self._h, req)

    def kv_table_blocks(self, req: int):
        """None if the request does not exist, else dict(ids, slots, states, len, resident)."""
        ids, slots, states = ((C.c_int32 * self._cap)() for _ in range(3))
        n, info = C.c_int32(0), (C.c_int32 * 2)()
        rc = lib.kv_table_blocks(self._h, req, ids, slots, states, self._cap, C.byref(n), info)
        if rc != KV_OK:
            return None
        k = n.value
        return dict(ids=list(ids[:k]), slots=list(slots[:k]), states=list(states[:k]), len=info[0],
                    resident=bool(info[1]))

    def kv_table_get_counts(self) -> dict:
        c = kv_table_counts()
        rc = lib.kv_table_get_counts(self._h, C.byref(c))
        if rc != KV_OK:
            raise KVError(rc, "kv_table_get_counts")
        return {f: getattr(c, f) for f, _ in kv_table_counts._fields_}

    def kv_table_destroy(self) -> int:
        if self._h:
            rc = lib.kv_table_destroy(self._h)
            self._h = C.c_void_p()
            return rc
        return KV_OK

    def __del__(self):
        try:
            self.kv_table_destroy()
        except Exception:
            pass
