"""ctypes loader for the plain-C oracle in duplexkv_oracle.c.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this module,
and this module imports nothing from the product package.

All arithmetic lives in the C file; this wrapper only marshals arguments.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "duplexkv_oracle.c")
_LIB = os.path.join(_HERE, "libduplexkv_oracle.so")

OK, EINVAL, ERANGE, EDUP, EOVERLAP, ENOSPC = 0, -1, -2, -3, -4, -8
NONE, DIRTY, FULL, SYNCED, HOST = 0, 1, 2, 3, 4   # block states of the table
BLOCK_FIRST, LAYER_FIRST = 0, 1            # host pool layouts
HBM_LAYER_FIRST, HBM_BLOCK_FIRST = 0, 1    # cache layouts


class OkvSchedParams(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("alpha", "beta_b", "beta_f", "slo_tbt", "slo_ttft")]


class OkvSchedReq(C.Structure):
    _fields_ = [("id", C.c_int32), ("state", C.c_int32), ("blocks", C.c_int32), ("pad", C.c_int32),
                ("t_ref", C.c_double)]


RUNNING, WAITING, ROTARY = 0, 1, 2


class OkvShape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "n_kv_heads", "head_dim", "block_size", "elem_bytes",
        "n_hbm_blocks", "n_host_slots", "host_layout", "hbm_layout")]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no HIP, no GPU)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-Werror",
                               "-shared", "-fPIC", "-pthread", "-o", _LIB, _SRC])
    return _LIB


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        p32 = C.POINTER(C.c_int32)
        ps = C.POINTER(OkvShape)
        for name in ("okv_seg_bytes", "okv_block_bytes", "okv_cache_bytes", "okv_pool_bytes"):
            getattr(L, name).restype = C.c_uint64
            getattr(L, name).argtypes = [ps]
        for name in ("okv_hbm_offset", "okv_pool_offset"):
            getattr(L, name).restype = C.c_uint64
            getattr(L, name).argtypes = [ps, C.c_int32, C.c_int32, C.c_int32]
        L.okv_validate.restype = C.c_int
        L.okv_validate.argtypes = [ps, p32, p32, C.c_int32, p32, p32, C.c_int32]
        L.okv_rotate.restype = C.c_int
        L.okv_rotate.argtypes = [ps, C.c_void_p, C.c_void_p, p32, p32, C.c_int32,
                                 p32, p32, C.c_int32]
        L.okv_rotate_threads.restype = C.c_int
        L.okv_rotate_threads.argtypes = L.okv_rotate.argtypes + [C.c_int32]
        L.okv_swap_out.restype = C.c_int
        L.okv_swap_out.argtypes = [ps, C.c_void_p, C.c_void_p, p32, p32, C.c_int32]
        L.okv_swap_in.restype = C.c_int
        L.okv_swap_in.argtypes = [ps, C.c_void_p, C.c_void_p, p32, p32, C.c_int32]
        L.okvt_create.restype = C.c_void_p
        L.okvt_create.argtypes = [ps, C.c_int32]
        L.okvt_destroy.restype = None
        L.okvt_destroy.argtypes = [C.c_void_p]
        L.okvt_append.restype = C.c_int
        L.okvt_append.argtypes = [C.c_void_p, C.c_int32, C.c_int32, p32, C.c_int32, p32]
        L.okvt_eager.restype = C.c_int
        L.okvt_eager.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, p32]
        L.okvt_rotate.restype = C.c_int
        L.okvt_rotate.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, p32, C.c_int32, p32, C.c_int32]
        L.okvt_rotate_eager.restype = C.c_int
        L.okvt_rotate_eager.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, p32, C.c_int32, p32, C.c_int32,
                                        C.c_int32, p32]
        L.okvt_finish.restype = C.c_int
        L.okvt_finish.argtypes = [C.c_void_p, C.c_int32]
        L.okvt_blocks.restype = C.c_int
        L.okvt_blocks.argtypes = [C.c_void_p, C.c_int32, p32, p32, p32, C.c_int32, p32, p32]
        L.okvt_counts.restype = C.c_int
        L.okvt_counts.argtypes = [C.c_void_p, C.POINTER(C.c_int64)]
        L.okv_sched_vlt.restype = C.c_double
        L.okv_sched_vlt.argtypes = [C.POINTER(OkvSchedParams), C.POINTER(OkvSchedReq), C.c_double]
        L.okv_sched_lvf.restype = C.c_int
        L.okv_sched_lvf.argtypes = [C.POINTER(OkvSchedParams), C.POINTER(OkvSchedReq), C.c_int32, C.c_double,
                                    C.c_int32, C.c_int32, p32, p32, p32, p32, p32]
        L.okv_read_checksum.restype = C.c_int
        L.okv_read_checksum.argtypes = [ps, C.c_void_p, p32, C.c_int32, C.POINTER(C.c_uint64)]
        _lib = L
    return _lib


def make_shape(n_layers, n_kv_heads, head_dim, block_size, n_hbm_blocks, n_host_slots,
               elem_bytes=2, host_layout=BLOCK_FIRST, hbm_layout=HBM_LAYER_FIRST) -> OkvShape:
    return OkvShape(n_layers, n_kv_heads, head_dim, block_size, elem_bytes,
                    n_hbm_blocks, n_host_slots, host_layout, hbm_layout)


def shape_of(kvshape, host_layout=BLOCK_FIRST, hbm_layout=HBM_LAYER_FIRST) -> OkvShape:
    """From any object with the KV shape attributes (e.g. workloads.KVShape)."""
    return make_shape(kvshape.n_layers, kvshape.n_kv_heads, kvshape.head_dim,
                      kvshape.block_size, kvshape.n_hbm_blocks, kvshape.n_host_slots,
                      kvshape.elem_bytes, host_layout, hbm_layout)


def _ids(a):
    """(pointer, n, keepalive) for an id list; None or empty gives (NULL, 0)."""
    if a is None:
        return None, 0, None
    arr = np.ascontiguousarray(a, dtype=np.int32)
    if arr.size == 0:
        return None, 0, arr
    return arr.ctypes.data_as(C.POINTER(C.c_int32)), int(arr.size), arr


def _buf(a) -> C.c_void_p:
    if a is None:
        return C.c_void_p(0)
    assert isinstance(a, np.ndarray) and a.dtype == np.uint8 and a.flags["C_CONTIGUOUS"]
    return C.c_void_p(a.ctypes.data)


def seg_bytes(s): return int(lib().okv_seg_bytes(C.byref(s)))
def block_bytes(s): return int(lib().okv_block_bytes(C.byref(s)))
def cache_bytes(s): return int(lib().okv_cache_bytes(C.byref(s)))
def pool_bytes(s): return int(lib().okv_pool_bytes(C.byref(s)))
def hbm_offset(s, l, kv, b): return int(lib().okv_hbm_offset(C.byref(s), l, kv, b))
def pool_offset(s, l, kv, sl): return int(lib().okv_pool_offset(C.byref(s), l, kv, sl))


def validate(s, out_ids, out_slots, in_ids, in_slots, n_out=None, n_in=None) -> int:
    po, no, k1 = _ids(out_ids); ps_, no2, k2 = _ids(out_slots)
    pi, ni, k3 = _ids(in_ids); pis, ni2, k4 = _ids(in_slots)
    assert no == no2 and ni == ni2, "id and slot lists of one direction differ in length"
    return lib().okv_validate(C.byref(s), po, ps_, no if n_out is None else n_out,
                              pi, pis, ni if n_in is None else n_in)


def rotate(s, hbm, pool, out_ids, out_slots, in_ids, in_slots, threads: int = 0) -> int:
    """In place on the uint8 images `hbm` and `pool`.  Returns the result code."""
    po, no, k1 = _ids(out_ids); ps_, no2, k2 = _ids(out_slots)
    pi, ni, k3 = _ids(in_ids); pis, ni2, k4 = _ids(in_slots)
    assert no == no2 and ni == ni2
    if hbm is not None:
        assert hbm.size == cache_bytes(s)
    if pool is not None:
        assert pool.size == pool_bytes(s)
    if threads > 0:
        return lib().okv_rotate_threads(C.byref(s), _buf(hbm), _buf(pool), po, ps_, no,
                                        pi, pis, ni, threads)
    return lib().okv_rotate(C.byref(s), _buf(hbm), _buf(pool), po, ps_, no, pi, pis, ni)


def swap_out(s, hbm, pool, ids, slots) -> int:
    pi, n, k1 = _ids(ids); psl, n2, k2 = _ids(slots)
    assert n == n2
    return lib().okv_swap_out(C.byref(s), _buf(hbm), _buf(pool), pi, psl, n)


def swap_in(s, hbm, pool, slots, ids) -> int:
    psl, n, k1 = _ids(slots); pi, n2, k2 = _ids(ids)
    assert n == n2
    return lib().okv_swap_in(C.byref(s), _buf(hbm), _buf(pool), psl, pi, n)


def read_checksum(s, hbm, ids):
    """(code, sum of all 32-bit words of the named blocks modulo 2**64)."""
    pi, n, k1 = _ids(ids)
    out = C.c_uint64(0)
    rc = lib().okv_read_checksum(C.byref(s), _buf(hbm), pi, n, C.byref(out))
    return rc, int(out.value)


COUNT_NAMES = ("free_hbm", "free_slots", "copied_eager", "copied_preempt", "dropped_synced", "swapped_in")


class Table:
    """The oracle's block table with eager rotation, over caller-held images."""

    def __init__(self, s, max_requests):
        self.s = s
        self._h = lib().okvt_create(C.byref(s), max_requests)
        assert self._h

    def append(self, req, n_tokens):
        """(code, [newly allocated HBM ids])."""
        cap = int(self.s.n_hbm_blocks)
        ids = (C.c_int32 * cap)()
        n = C.c_int32(0)
        rc = lib().okvt_append(self._h, req, n_tokens, ids, cap, C.byref(n))
        return rc, [ids[i] for i in range(n.value)] if rc == OK else []

    def eager(self, hbm, pool, budget):
        n = C.c_int32(0)
        rc = lib().okvt_eager(self._h, _buf(hbm), _buf(pool), budget, C.byref(n))
        return rc, n.value

    def rotate(self, hbm, pool, preempt, resume):
        pp, np_, k1 = _ids(preempt)
        pr, nr, k2 = _ids(resume)
        return lib().okvt_rotate(self._h, _buf(hbm), _buf(pool), pp, np_, pr, nr)

    def rotate_eager(self, hbm, pool, preempt, resume, budget):
        pp, np_, k1 = _ids(preempt)
        pr, nr, k2 = _ids(resume)
        n = C.c_int32(0)
        rc = lib().okvt_rotate_eager(self._h, _buf(hbm), _buf(pool), pp, np_, pr, nr, budget, C.byref(n))
        return rc, n.value

    def finish(self, req):
        return lib().okvt_finish(self._h, req)

    def blocks(self, req):
        """None if the request does not exist, else dict(ids, slots, states, len, resident)."""
        cap = int(self.s.n_hbm_blocks)
        ids, slots, states = (C.c_int32 * cap)(), (C.c_int32 * cap)(), (C.c_int32 * cap)()
        n, info = C.c_int32(0), (C.c_int32 * 2)()
        rc = lib().okvt_blocks(self._h, req, ids, slots, states, cap, C.byref(n), info)
        if rc != OK:
            return None
        k = n.value
        return dict(ids=list(ids[:k]), slots=list(slots[:k]), states=list(states[:k]), len=info[0],
                    resident=bool(info[1]))

    def counts(self):
        c = (C.c_int64 * 8)()
        assert lib().okvt_counts(self._h, c) == OK
        return dict(zip(COUNT_NAMES, c[:6]))

    def close(self):
        if self._h:
            lib().okvt_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()


def sched_vlt(params, req, t_now):
    """params = (alpha, beta_b, beta_f, slo_tbt, slo_ttft); req = (id, state, blocks, t_ref)."""
    p = OkvSchedParams(*params)
    r = OkvSchedReq(req[0], req[1], req[2], 0, req[3])
    return lib().okv_sched_vlt(C.byref(p), C.byref(r), t_now)


def sched_lvf(params, reqs, t_now, b_xfer, b_hbm):
    """(code, preempted ids, prioritised ids, fcfs flag)."""
    p = OkvSchedParams(*params)
    n = len(reqs)
    arr = (OkvSchedReq * max(n, 1))(*[OkvSchedReq(r[0], r[1], r[2], 0, r[3]) for r in reqs])
    pre, pri = (C.c_int32 * max(n, 1))(), (C.c_int32 * max(n, 1))()
    npre, npri, fcfs = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    rc = lib().okv_sched_lvf(C.byref(p), arr, n, t_now, b_xfer, b_hbm, pre, C.byref(npre), pri, C.byref(npri),
                             C.byref(fcfs))
    return rc, list(pre[:npre.value]), list(pri[:npri.value]), bool(fcfs.value)
